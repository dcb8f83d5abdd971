// Measurement aids (include/dlprobe.h): a register-resident MFMA loop and plain streaming
// kernels.  They compute nothing of the method; the benchmark runs them beside the real kernels
// to show what the matrix units and the memory system give on the box at hand.
#include <hip/hip_runtime.h>

#include "../../include/dlprobe.h"
#include "device_common.h"
#include "kernels.h"

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lcg(uint32_t &s)
{
    s = s * 1664525u + 1013904223u;
    return s;
}
// Sum of six uniforms, centred and scaled to unit variance: close enough to a normal for a power test.
__device__ __forceinline__ float near_normal(uint32_t &s)
{
    float t = 0.f;
    for (int i = 0; i < 6; ++i) t += (float)(lcg(s) >> 8) * (1.0f / 16777216.0f);
    return (t - 3.0f) * 1.41421356f;
}

template <int SHAPE, int OPERANDS>
__global__ __launch_bounds__(256) void mfma_loop_kernel(float *__restrict__ sink, unsigned long long *__restrict__ clocks, int iters)
{
    half8_t a[4], b[4];
    uint32_t s = threadIdx.x * 7919u + blockIdx.x * 104729u + 1u;
    for (int r = 0; r < 4; ++r)
        for (int i = 0; i < 8; ++i) {
            if (OPERANDS == 0) {
                a[r][i] = (_Float16)1.0f;
                b[r][i] = (_Float16)0.5f;
            } else {
                a[r][i] = (_Float16)fabsf(near_normal(s));
                b[r][i] = (_Float16)(0.03f * near_normal(s));
            }
        }
    const unsigned long long w0 = wall_clock64(), c0 = clock64();
    float total = 0.f;
    if (SHAPE == 0) {
        f32x16_t c[4];
        for (int u = 0; u < 4; ++u)
            for (int i = 0; i < 16; ++i) c[u][i] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                c[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(u + (u >> 2)) & 3], b[(u + 2 * (u >> 2)) & 3], c[u & 3], 0, 0, 0);
        }
        for (int u = 0; u < 4; ++u)
            for (int i = 0; i < 16; ++i) total += c[u][i];
    } else {
        f32x4_t c[16];
        for (int u = 0; u < 16; ++u) c[u] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 16; ++u)
                c[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u & 3], b[(u + (u >> 2)) & 3], c[u], 0, 0, 0);
        }
        for (int u = 0; u < 16; ++u) total += c[u][0] + c[u][1] + c[u][2] + c[u][3];
    }
    const unsigned long long w1 = wall_clock64(), c1 = clock64();
    sink[blockIdx.x * 256 + threadIdx.x] = total;
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        clocks[0] = w1 - w0;
        clocks[1] = c1 - c0;
    }
}

// A wavefront moves whole 3 KB trips (three 1 KB rows, lane i chunk i of each), as the loss kernel does.
template <int MODE>
__global__ __launch_bounds__(256) void stream_kernel(const dlk::u32x4_t *__restrict__ src, const dlk::u32x2_t *__restrict__ aux,
                                                     dlk::u32x4_t *__restrict__ dst, int64_t trips, uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int64_t first = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), stride = (int64_t)gridDim.x * 4;
    dlk::u32x4_t acc{0, 0, 0, 0};
    for (int64_t t = first; t < trips; t += stride) {
        dlk::u32x4_t v0{(uint32_t)t, 1, 2, 3}, v1 = v0, v2 = v0;
        if (MODE != 2) {
            const dlk::u32x4_t *p = src + t * 192;
            v0 = __builtin_nontemporal_load(p + lane);
            v1 = __builtin_nontemporal_load(p + 64 + lane);
            v2 = __builtin_nontemporal_load(p + 128 + lane);
        }
        if (MODE == 3) {
            const dlk::u32x2_t l = aux[t * 64 + lane];
            v0[0] ^= l[0];
            v1[1] ^= l[1];
        }
        if (MODE == 0) {
            acc[0] ^= v0[0] ^ v1[1] ^ v2[2];
            acc[1] ^= v0[3] ^ v1[0] ^ v2[1];
        } else {
            dlk::u32x4_t *q = dst + t * 192;
            __builtin_nontemporal_store(v0, q + lane);
            __builtin_nontemporal_store(v1, q + 64 + lane);
            __builtin_nontemporal_store(v2, q + 128 + lane);
        }
    }
    if (MODE == 0 && acc[0] == 0x12345678u && acc[1] == 77u) sink[0] = acc[0];
}

}  // namespace

extern "C" {

int dl_probe_mfma(int32_t shape, int32_t operands, int32_t iters, float *sink, uint64_t *clocks, double *flop, void *hip_stream)
{
    if (!sink || !clocks || !flop) return 1;
    if ((shape != 0 && shape != 1) || (operands != 0 && operands != 1) || iters < 1) return 2;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long *clk = reinterpret_cast<unsigned long long *>(clocks);
    const dim3 grid(1024), block(256);
    if (shape == 0 && operands == 0) hipLaunchKernelGGL((mfma_loop_kernel<0, 0>), grid, block, 0, stream, sink, clk, iters);
    else if (shape == 0) hipLaunchKernelGGL((mfma_loop_kernel<0, 1>), grid, block, 0, stream, sink, clk, iters);
    else if (operands == 0) hipLaunchKernelGGL((mfma_loop_kernel<1, 0>), grid, block, 0, stream, sink, clk, iters);
    else hipLaunchKernelGGL((mfma_loop_kernel<1, 1>), grid, block, 0, stream, sink, clk, iters);
    *flop = 1024.0 * 4.0 * (double)iters * 262144.0;
    return hipGetLastError() == hipSuccess ? 0 : 7;
}

int dl_probe_stream(int32_t mode, const void *src, const void *aux, void *dst, int64_t bytes, uint32_t *sink, void *hip_stream)
{
    if (mode < 0 || mode > 3 || bytes < 0 || bytes % 3072 != 0) return 2;
    if (!sink || (mode != 2 && !src) || (mode != 0 && !dst) || (mode == 3 && !aux)) return 1;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(aux)) & 15u) return 2;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t trips = bytes / 3072;
    const dim3 grid(1024), block(256);
    const dlk::u32x4_t *s = static_cast<const dlk::u32x4_t *>(src);
    const dlk::u32x2_t *a = static_cast<const dlk::u32x2_t *>(aux);
    dlk::u32x4_t *d = static_cast<dlk::u32x4_t *>(dst);
    if (mode == 0) hipLaunchKernelGGL(stream_kernel<0>, grid, block, 0, stream, s, a, d, trips, sink);
    else if (mode == 1) hipLaunchKernelGGL(stream_kernel<1>, grid, block, 0, stream, s, a, d, trips, sink);
    else if (mode == 2) hipLaunchKernelGGL(stream_kernel<2>, grid, block, 0, stream, s, a, d, trips, sink);
    else hipLaunchKernelGGL(stream_kernel<3>, grid, block, 0, stream, s, a, d, trips, sink);
    return hipGetLastError() == hipSuccess ? 0 : 7;
}

}  // extern "C"
