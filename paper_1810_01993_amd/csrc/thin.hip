// Streaming kernels for 1x1 convolutions with a handful of channels on one
// side (the 3-class logits layer): there the data gradient and the filter
// gradient are bandwidth-bound outer-product / dot-product sweeps over the
// 256-channel activation tensor, and an MFMA tile padded from 3 to 32 would
// only add latency.
#include "device_common.h"
#include "kernels.h"

namespace dlk {

constexpr int THIN_MAX = 4;      // channels on the thin side

// D[m][j..j+7] = sum_{c < Cin} A[m][c] * B[j..j+7][c]   (one tap, dense rows, Cin <= THIN_MAX, Nout % 8 == 0)
// A thread owns one group of 8 output columns and keeps their filter values in registers.  A workgroup owns a
// contiguous range of rows, fetches their A values (Cin per row) coalesced into LDS, SUB rows at a time, and
// walks down them: one 16-byte store per Cin LDS broadcast reads, no global load between two stores (with the
// A values read from memory row by row the sweep took 0.30 instead of 0.23 ms on the logits layer whenever
// other kernels had run since the last call, as in a training step).
template <class T>
__global__ __launch_bounds__(256) void thin_rows_kernel(const IgemmArgs p)
{
    constexpr int SUB = 512;
    __shared__ float sa[SUB * THIN_MAX];
    const int groups = p.Nout / 8;
    const int gpb = groups < 256 ? groups : 256;
    const int rows_pb = 256 / gpb;
    const int g = blockIdx.y * gpb + threadIdx.x % gpb, r = threadIdx.x / gpb;
    const bool active = r < rows_pb && g < groups;
    const int j = active ? g * 8 : 0;
    float b[8][THIN_MAX];
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int c = 0; c < THIN_MAX; ++c) b[e][c] = c < p.Cin ? T::to_float(p.B[(size_t)(j + e) * p.Cin + c]) : 0.f;
    const int64_t M = (int64_t)p.NB * p.OH * p.OW;
    const int64_t chunk = (M + gridDim.x - 1) / gridDim.x;
    const int64_t m_begin = (int64_t)blockIdx.x * chunk, m_end = m_begin + chunk < M ? m_begin + chunk : M;
    for (int64_t sub = m_begin; sub < m_end; sub += SUB) {
        const int n = (int)(m_end - sub < SUB ? m_end - sub : SUB);
        __syncthreads();
        for (int i = threadIdx.x; i < n * p.Cin; i += 256) {
            const int row = i / p.Cin, c = i - row * p.Cin;
            sa[row * THIN_MAX + c] = T::to_float(p.A[sub * p.Cin + i]);
        }
        __syncthreads();
        if (!active) continue;
#pragma unroll 4
        for (int q = r; q < n; q += rows_pb) {
            const int64_t m = sub + q;
            float a[THIN_MAX];
#pragma unroll
            for (int c = 0; c < THIN_MAX; ++c) a[c] = c < p.Cin ? sa[q * THIN_MAX + c] : 0.f;
            u32x4_t out, rv{0, 0, 0, 0};
            if (p.resid) rv = *reinterpret_cast<const u32x4_t *>(p.resid + m * p.ldd + j);
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                float s0 = T::to_float((uint16_t)(rv[e >> 1] & 0xffffu)), s1 = T::to_float((uint16_t)(rv[e >> 1] >> 16));
#pragma unroll
                for (int c = 0; c < THIN_MAX; ++c) {
                    s0 += a[c] * b[e][c];
                    s1 += a[c] * b[e + 1][c];
                }
                s0 = apply_tail(s0, p.bias, p.relu, j + e);
                s1 = apply_tail(s1, p.bias, p.relu, j + e + 1);
                out[e >> 1] = (uint32_t)T::from_float(s0) | ((uint32_t)T::from_float(s1) << 16);
            }
            __builtin_nontemporal_store(out, reinterpret_cast<u32x4_t *>(p.D + m * p.ldd + j));
        }
    }
}

bool thin_rows_applicable(const IgemmArgs &a)
{
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW &&
                       a.IH == a.OH && a.IW == a.OW;
    return dense && a.TR == 1 && a.TS == 1 && a.th0 == 0 && a.tw0 == 0 && a.Cin <= THIN_MAX && a.Nout % 8 == 0 &&
           a.ldd % 8 == 0;
}

hipError_t launch_thin_rows(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    const int groups = a.Nout / 8;
    if (M <= 0 || groups <= 0) return hipSuccess;
    const int gpb = groups < 256 ? groups : 256, rows_pb = 256 / gpb;
    // 512 rows per workgroup (best of 64..4096 on the logits layer); fewer when that would leave compute units idle
    int64_t per = (M + 1023) / 1024;
    per = (per + rows_pb - 1) / rows_pb * rows_pb;
    if (per < 4 * rows_pb) per = 4 * rows_pb;
    if (per > 512) per = 512;
    const int64_t wg = (M + per - 1) / per;
    const dim3 grid((unsigned)(wg < 65535 ? wg : 65535), (unsigned)((groups + gpb - 1) / gpb)), block(256);
    if (is_bf16) DLK_LAUNCH("thin_rows_kernel", thin_rows_kernel<BF16>, grid, block, 0, stream, a);
    else DLK_LAUNCH("thin_rows_kernel", thin_rows_kernel<F16>, grid, block, 0, stream, a);
    return dlk::launch_status();
}

// Filter gradient of a 1x1, stride-1, unpadded convolution with K <= THIN_MAX:
//   partial[b][k][c] = sum over workgroup b's pixels of dy[pix][k] * x[pix][c].
// A workgroup is (C/8 channel groups) x (256 / (C/8) pixel lanes); every thread
// keeps K x 8 running sums, the pixel lanes are then added in a fixed order.
// The workgroup's slice of dy is staged in LDS as fp32, 512 pixels at a time, so
// that the inner loop issues one 16-byte global load per pixel and nothing else.
template <class T>
__global__ __launch_bounds__(256) void thin_wgrad_kernel(const WgradArgs p)
{
    constexpr int SUB = 512;                             // pixels of dy staged at a time
    __shared__ float red[256 * 8];                       // 8 sums per thread, reused for each k
    __shared__ float sdy[SUB * THIN_MAX];
    const int groups = p.C / 8;                          // <= 256
    const int lanes = 256 / groups;                      // pixel lanes per workgroup
    const int g = threadIdx.x % groups, pl = threadIdx.x / groups;
    const int npix = p.N * p.P * p.Q;
    const int pix_begin = blockIdx.x * p.chunk, pix_end = min(npix, pix_begin + p.chunk);
    float acc[THIN_MAX][8];
#pragma unroll
    for (int k = 0; k < THIN_MAX; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    for (int sub = pix_begin; sub < pix_end; sub += SUB) {
        const int sub_end = min(pix_end, sub + SUB);
        __syncthreads();                                 // the previous part of dy is no longer read
        for (int i = threadIdx.x; i < (sub_end - sub) * p.K; i += 256) {
            const int px = i / p.K, k = i - px * p.K;
            sdy[px * THIN_MAX + k] = T::to_float(p.dy[(size_t)sub * p.K + i]);
        }
        __syncthreads();
        if (pl < lanes) {
#pragma unroll 4
            for (int pix = sub + pl; pix < sub_end; pix += lanes) {
                const u32x4_t xv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p.x + (size_t)pix * p.C + g * 8));
                float xf[8];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    xf[2 * d] = T::to_float((uint16_t)(xv[d] & 0xffffu));
                    xf[2 * d + 1] = T::to_float((uint16_t)(xv[d] >> 16));
                }
                const float *gd = sdy + (pix - sub) * THIN_MAX;
#pragma unroll
                for (int k = 0; k < THIN_MAX; ++k)
                    if (k < p.K) {
                        const float gk = gd[k];
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[k][e] += gk * xf[e];
                    }
            }
        }
    }
    float *out = p.partial + (size_t)blockIdx.x * p.K * p.C;
    for (int k = 0; k < p.K; ++k) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = 0.f;
#pragma unroll
            for (int kk = 0; kk < THIN_MAX; ++kk) if (kk == k) v = acc[kk][e];
            red[threadIdx.x * 8 + e] = (pl < lanes) ? v : 0.f;
        }
        __syncthreads();
        if (pl == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float s = 0.f;
                for (int l = 0; l < lanes; ++l) s += red[(l * groups + g) * 8 + e];
                out[(size_t)k * p.C + g * 8 + e] = s;
            }
        }
    }
}

bool thin_wgrad_applicable(int K, int C, int R, int S, int sh, int sw, int ph, int pw)
{
    return K <= THIN_MAX && R == 1 && S == 1 && sh == 1 && sw == 1 && ph == 0 && pw == 0 && C % 8 == 0 && C / 8 <= 256 &&
           C >= 8;
}

hipError_t launch_thin_wgrad(const WgradArgs &a, bool is_bf16, hipStream_t stream)
{
    const dim3 grid((unsigned)a.splits), block(256);
    if (is_bf16) DLK_LAUNCH("thin_wgrad_kernel", thin_wgrad_kernel<BF16>, grid, block, 0, stream, a);
    else DLK_LAUNCH("thin_wgrad_kernel", thin_wgrad_kernel<F16>, grid, block, 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
