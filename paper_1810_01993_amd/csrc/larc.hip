// LARC weight update (layer-wise adaptive rate control) for many tensors in two launches.
//
// Per tensor t with fp32 weights w, gradient g (fp16, bf16 or fp32) and optional fp32 momentum
// buffer v:
//     local = trust * ||w|| / (||g|| + wd * ||w|| + eps)      (lr itself if ||w|| or ||g|| is 0)
//     rate  = clip ? min(local, lr) : local * lr
//     v    <- momentum * v + rate * (g + wd * w);   w <- w - v
// Launch 1 (grid: slices x tensors): every workgroup adds w^2 and g^2 over its slice of its
// tensor (fp32, fixed order) and writes two partial sums.  Launch 2 (same grid): every
// workgroup adds its tensor's partials in ascending slice order (so all of them derive the very
// same rate), then updates its slice.  The tensor table travels as a kernel argument (no
// device-side table to upload), at most LARC_MAX tensors per pair of launches.
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

constexpr int LARC_THREADS = 256;

template <class G> __device__ __forceinline__ float larc_grad(const void *g, int64_t i);
template <> __device__ __forceinline__ float larc_grad<F16>(const void *g, int64_t i) { return F16::to_float(static_cast<const uint16_t *>(g)[i]); }
template <> __device__ __forceinline__ float larc_grad<BF16>(const void *g, int64_t i) { return BF16::to_float(static_cast<const uint16_t *>(g)[i]); }
template <> __device__ __forceinline__ float larc_grad<float>(const void *g, int64_t i) { return static_cast<const float *>(g)[i]; }

// four consecutive gradient values starting at element i (i % 4 == 0, tensor base suitably aligned)
template <class G> __device__ __forceinline__ floatx4_t larc_grad4(const void *g, int64_t i)
{
    if constexpr (std::is_same<G, float>::value) {
        return *reinterpret_cast<const floatx4_t *>(static_cast<const float *>(g) + i);
    } else {
        const u32x2_t v = *reinterpret_cast<const u32x2_t *>(static_cast<const uint16_t *>(g) + i);
        return floatx4_t{G::to_float((uint16_t)(v[0] & 0xffffu)), G::to_float((uint16_t)(v[0] >> 16)),
                         G::to_float((uint16_t)(v[1] & 0xffffu)), G::to_float((uint16_t)(v[1] >> 16))};
    }
}
// 16-byte accesses are possible when the tensor's bases allow it (slices start at multiples of 4 elements)
template <class G> __device__ __forceinline__ bool larc_vec_ok(const LarcTensor &t)
{
    const uintptr_t gmask = std::is_same<G, float>::value ? 15u : 7u;
    return ((reinterpret_cast<uintptr_t>(t.w) | reinterpret_cast<uintptr_t>(t.v)) & 15u) == 0 &&
           (reinterpret_cast<uintptr_t>(t.g) & gmask) == 0;
}

__device__ __forceinline__ void larc_slice(int64_t count, int64_t *begin, int64_t *end)
{
    const int64_t chunk = ((count + LARC_SLICES - 1) / LARC_SLICES + 3) / 4 * 4;
    *begin = min(count, (int64_t)blockIdx.x * chunk);
    *end = min(count, *begin + chunk);
}

template <class G>
__global__ __launch_bounds__(LARC_THREADS) void larc_norm_kernel(const LarcBatch b)
{
    const LarcTensor &t = b.t[blockIdx.y];
    int64_t begin, end;
    larc_slice(t.count, &begin, &end);
    float sw = 0.f, sg = 0.f;
    int64_t i0 = begin;
    if (larc_vec_ok<G>(t)) {
        const int64_t vend = begin + (end - begin) / 4 * 4;
        for (int64_t i = begin + 4 * threadIdx.x; i < vend; i += 4 * LARC_THREADS) {
            const floatx4_t w = *reinterpret_cast<const floatx4_t *>(t.w + i), g = larc_grad4<G>(t.g, i);
            sw += (w[0] * w[0] + w[1] * w[1]) + (w[2] * w[2] + w[3] * w[3]);
            sg += (g[0] * g[0] + g[1] * g[1]) + (g[2] * g[2] + g[3] * g[3]);
        }
        i0 = vend;
    }
    for (int64_t i = i0 + threadIdx.x; i < end; i += LARC_THREADS) {
        const float w = t.w[i], g = larc_grad<G>(t.g, i);
        sw += w * w;
        sg += g * g;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sw += __shfl_down(sw, off, 64);
        sg += __shfl_down(sg, off, 64);
    }
    __shared__ float red[2][LARC_THREADS / 64];
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = sw; red[1][threadIdx.x >> 6] = sg; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float *out = b.partial + ((size_t)(b.first + blockIdx.y) * LARC_SLICES + blockIdx.x) * 2;
        out[0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        out[1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

template <class G>
__global__ __launch_bounds__(LARC_THREADS) void larc_update_kernel(const LarcBatch b)
{
    const LarcTensor &t = b.t[blockIdx.y];
    __shared__ float s_rate;
    if (threadIdx.x == 0) {
        const float *p = b.partial + (size_t)(b.first + blockIdx.y) * LARC_SLICES * 2;
        float sw = 0.f, sg = 0.f;
        for (int i = 0; i < LARC_SLICES; ++i) { sw += p[2 * i]; sg += p[2 * i + 1]; }
        const float wn = sqrtf(sw), gn = sqrtf(sg);
        const float local = (wn > 0.f && gn > 0.f) ? b.trust * wn / (gn + b.wd * wn + b.eps) : (b.clip ? b.lr : 1.f);
        const float rate = b.clip ? fminf(local, b.lr) : local * b.lr;
        s_rate = rate;
        if (blockIdx.x == 0 && b.rates) b.rates[b.first + blockIdx.y] = rate;
    }
    __syncthreads();
    const float rate = s_rate;
    int64_t begin, end;
    larc_slice(t.count, &begin, &end);
    int64_t i0 = begin;
    if (larc_vec_ok<G>(t)) {
        const int64_t vend = begin + (end - begin) / 4 * 4;
        for (int64_t i = begin + 4 * threadIdx.x; i < vend; i += 4 * LARC_THREADS) {
            const floatx4_t w = *reinterpret_cast<const floatx4_t *>(t.w + i), g = larc_grad4<G>(t.g, i);
            floatx4_t step;
#pragma unroll
            for (int e = 0; e < 4; ++e) step[e] = rate * (g[e] + b.wd * w[e]);
            if (t.v) {
                const floatx4_t v = *reinterpret_cast<const floatx4_t *>(t.v + i);
#pragma unroll
                for (int e = 0; e < 4; ++e) step[e] += b.momentum * v[e];
                *reinterpret_cast<floatx4_t *>(t.v + i) = step;
            }
            *reinterpret_cast<floatx4_t *>(t.w + i) = w - step;
        }
        i0 = vend;
    }
    for (int64_t i = i0 + threadIdx.x; i < end; i += LARC_THREADS) {
        const float w = t.w[i];
        float step = rate * (larc_grad<G>(t.g, i) + b.wd * w);
        if (t.v) {
            step += b.momentum * t.v[i];
            t.v[i] = step;
        }
        t.w[i] = w - step;
    }
}

template <class G>
static hipError_t larc_launch(const LarcBatch &b, hipStream_t stream)
{
    const dim3 grid(LARC_SLICES, (unsigned)b.n), block(LARC_THREADS);
    DLK_LAUNCH("larc_norm_kernel", larc_norm_kernel<G>, grid, block, 0, stream, b);
    hipError_t e = dlk::launch_status();
    if (e != hipSuccess) return e;
    DLK_LAUNCH("larc_update_kernel", larc_update_kernel<G>, grid, block, 0, stream, b);
    return dlk::launch_status();
}

hipError_t launch_larc(const LarcBatch &b, int grad_dtype, hipStream_t stream)
{
    if (b.n < 1 || b.n > LARC_MAX) return hipErrorInvalidValue;
    if (grad_dtype == 0) return larc_launch<F16>(b, stream);
    if (grad_dtype == 1) return larc_launch<BF16>(b, stream);
    return larc_launch<float>(b, stream);
}

}  // namespace dlk
