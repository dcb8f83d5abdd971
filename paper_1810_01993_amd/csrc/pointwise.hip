// Backward of the point-wise tail of a convolution layer, y = max(s + bias[k], 0), in one
// streaming pass over the [pixels][K] tensors:
//   dz[i][k]  = dy[i][k] where y[i][k] > 0, else 0     (the gradient the convolution's own
//                                                       data- and filter-gradient kernels take)
//   dbias[k]  = sum over pixels of dz[i][k]
// 6 bytes of traffic per element (dy and y in, dz out) instead of the 10 of a masking pass
// followed by a column-sum pass.  A thread owns VEC consecutive channels (8 = one 16-byte
// access, or 1 for channel counts that are not a multiple of 8) and walks down the pixels of
// its workgroup's slab with fp32 running sums; the pixel lanes of a workgroup are then added
// in a fixed order through LDS, every workgroup writes one fp32 partial row, and the ordered
// reduce kernel adds the rows: the result does not depend on timing.
#include "device_common.h"
#include "kernels.h"

namespace dlk {

constexpr int TB_THREADS = 256;

template <class T, int VEC>
__global__ __launch_bounds__(TB_THREADS) void tail_bwd_kernel(const TailBwdArgs p)
{
    __shared__ float red[TB_THREADS * VEC];
    const int groups_all = (p.K + VEC - 1) / VEC;                   // channel groups of the tensor
    const int gpb = groups_all < TB_THREADS ? groups_all : TB_THREADS;   // groups per workgroup
    const int lanes = TB_THREADS / gpb;                             // pixel lanes per workgroup
    const int gl = threadIdx.x % gpb, pl = threadIdx.x / gpb;
    const int g = blockIdx.y * gpb + gl;
    const bool active = pl < lanes && g < groups_all;
    const int k0 = g * VEC;
    const int64_t begin = (int64_t)blockIdx.x * p.chunk, end = min(p.npix, begin + p.chunk);
    float sum[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) sum[e] = 0.f;
    if (active) {
#pragma unroll 2
        for (int64_t i = begin + pl; i < end; i += lanes) {
            const size_t off = (size_t)i * p.K + k0;
            if constexpr (VEC == 8) {
                const u32x4_t gv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p.dy + off));
                u32x4_t out = gv;
                if (p.relu) {
                    const u32x4_t yv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p.y + off));
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t lo = T::to_float((uint16_t)(yv[d] & 0xffffu)) > 0.f ? 0xffffu : 0u;
                        const uint32_t hi = T::to_float((uint16_t)(yv[d] >> 16)) > 0.f ? 0xffff0000u : 0u;
                        out[d] = gv[d] & (lo | hi);
                    }
                    __builtin_nontemporal_store(out, reinterpret_cast<u32x4_t *>(p.dz + off));
                }
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    sum[2 * d] += T::to_float((uint16_t)(out[d] & 0xffffu));
                    sum[2 * d + 1] += T::to_float((uint16_t)(out[d] >> 16));
                }
            } else {
                if (k0 < p.K) {
                    uint16_t v = p.dy[off];
                    if (p.relu) {
                        if (!(T::to_float(p.y[off]) > 0.f)) v = 0;
                        p.dz[off] = v;
                    }
                    sum[0] += T::to_float(v);
                }
            }
        }
    }
    // pixel lanes added in ascending order
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[threadIdx.x * VEC + e] = active ? sum[e] : 0.f;
    __syncthreads();
    if (pl == 0 && g < groups_all) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float s = 0.f;
            for (int l = 0; l < lanes; ++l) s += red[(l * gpb + gl) * VEC + e];
            if (k0 + e < p.K) p.partial[(size_t)blockIdx.x * p.K + k0 + e] = s;
        }
    }
}

int tail_bwd_blocks(int64_t npix, int K)
{
    if (npix <= 0) return 1;
    const int vec = K % 8 == 0 ? 8 : 1;
    const int groups = (K + vec - 1) / vec, gpb = groups < TB_THREADS ? groups : TB_THREADS, lanes = TB_THREADS / gpb;
    int64_t b = (npix + (int64_t)lanes * 32 - 1) / ((int64_t)lanes * 32);     // about 32 pixels per thread
    if (b > 1024) b = 1024;
    return (int)(b < 1 ? 1 : b);
}

hipError_t launch_tail_bwd(const TailBwdArgs &a0, bool is_bf16, hipStream_t stream)
{
    TailBwdArgs a = a0;
    const int blocks = tail_bwd_blocks(a.npix, a.K);
    a.chunk = (a.npix + blocks - 1) / blocks;
    if (a.chunk < 1) a.chunk = 1;
    const int vec = a.K % 8 == 0 ? 8 : 1;
    const int groups = (a.K + vec - 1) / vec, gpb = groups < TB_THREADS ? groups : TB_THREADS;
    const dim3 grid((unsigned)blocks, (unsigned)((groups + gpb - 1) / gpb)), block(TB_THREADS);
    if (vec == 8) {
        if (is_bf16) DLK_LAUNCH("tail_bwd_kernel", (tail_bwd_kernel<BF16, 8>), grid, block, 0, stream, a);
        else DLK_LAUNCH("tail_bwd_kernel", (tail_bwd_kernel<F16, 8>), grid, block, 0, stream, a);
    } else {
        if (is_bf16) DLK_LAUNCH("tail_bwd_kernel", (tail_bwd_kernel<BF16, 1>), grid, block, 0, stream, a);
        else DLK_LAUNCH("tail_bwd_kernel", (tail_bwd_kernel<F16, 1>), grid, block, 0, stream, a);
    }
    hipError_t e = dlk::launch_status();
    if (e != hipSuccess) return e;
    return launch_splitk_reduce(a.partial, blocks, a.K, a.dbias, 2, stream);
}

}  // namespace dlk
