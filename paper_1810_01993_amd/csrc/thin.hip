// Streaming kernels for 1x1 convolutions with a handful of channels on one
// side (the 3-class logits layer): there the data gradient and the filter
// gradient are bandwidth-bound outer-product / dot-product sweeps over the
// 256-channel activation tensor, and an MFMA tile padded from 3 to 32 would
// only add latency.
#include <type_traits>

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
// CIN: the number of input channels (1..THIN_MAX) known at compile time; TAIL: bias, ReLU or a residual
// input present.  (With both read at run time the row loop held ~100 vector instructions and 16 branches
// per 16-byte store and the instruction issue, not memory, bounded the sweep.)
template <class T, int CIN, bool TAIL>
__global__ __launch_bounds__(256) void thin_rows_kernel(const IgemmArgs p)
{
    constexpr int SUB = 512;
    __shared__ __align__(16) float sa[SUB * THIN_MAX];
    const int groups = p.Nout / 8;
    const int gpb = groups < 256 ? groups : 256;
    const int rows_pb = 256 / gpb;
    const int g = blockIdx.y * gpb + threadIdx.x % gpb, r = threadIdx.x / gpb;
    const bool active = r < rows_pb && g < groups;
    const int j = active ? g * 8 : 0;
    float b[8][CIN];
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int c = 0; c < CIN; ++c) b[e][c] = T::to_float(p.B[(size_t)(j + e) * CIN + c]);
    const int64_t M = (int64_t)p.NB * p.OH * p.OW;
    const int64_t chunk = (M + gridDim.x - 1) / gridDim.x;
    const int64_t m_begin = (int64_t)blockIdx.x * chunk, m_end = m_begin + chunk < M ? m_begin + chunk : M;
    for (int64_t sub = m_begin; sub < m_end; sub += SUB) {
        const int n = (int)(m_end - sub < SUB ? m_end - sub : SUB);
        __syncthreads();
        for (int i = threadIdx.x; i < n * CIN; i += 256) {
            const int row = i / CIN, c = i - row * CIN;
            sa[row * THIN_MAX + c] = T::to_float(p.A[sub * CIN + i]);
        }
        __syncthreads();
        if (!active) continue;
        uint16_t *dst = p.D + (sub + r) * p.ldd + j;
        const size_t dstep = (size_t)rows_pb * p.ldd;
#pragma unroll 4
        for (int q = r; q < n; q += rows_pb, dst += dstep) {
            const floatx4_t a4 = *reinterpret_cast<const floatx4_t *>(sa + q * THIN_MAX);   // one 16-byte broadcast read
            u32x4_t out, rv{0, 0, 0, 0};
            if constexpr (TAIL)
                if (p.resid) rv = *reinterpret_cast<const u32x4_t *>(p.resid + (sub + q) * p.ldd + j);
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                float s0 = 0.f, s1 = 0.f;
                if constexpr (TAIL) {
                    s0 = T::to_float((uint16_t)(rv[e >> 1] & 0xffffu));
                    s1 = T::to_float((uint16_t)(rv[e >> 1] >> 16));
                }
#pragma unroll
                for (int c = 0; c < CIN; ++c) {
                    s0 += a4[c] * b[e][c];
                    s1 += a4[c] * b[e + 1][c];
                }
                if constexpr (TAIL) {
                    s0 = apply_tail(s0, p.bias, p.relu, j + e);
                    s1 = apply_tail(s1, p.bias, p.relu, j + e + 1);
                }
                out[e >> 1] = T::pack2(s0, s1);
            }
            __builtin_nontemporal_store(out, reinterpret_cast<u32x4_t *>(dst));
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
    const bool tail = a.bias || a.relu || a.resid;
    auto go = [&](auto cin, auto has_tail) {
        constexpr int CIN = decltype(cin)::value;
        constexpr bool TAIL = decltype(has_tail)::value;
        if (is_bf16) DLK_LAUNCH("thin_rows_kernel", (thin_rows_kernel<BF16, CIN, TAIL>), grid, block, 0, stream, a);
        else DLK_LAUNCH("thin_rows_kernel", (thin_rows_kernel<F16, CIN, TAIL>), grid, block, 0, stream, a);
    };
    auto by_tail = [&](auto cin) {
        if (tail) go(cin, std::true_type{});
        else go(cin, std::false_type{});
    };
    switch (a.Cin) {
        case 1: by_tail(std::integral_constant<int, 1>{}); break;
        case 2: by_tail(std::integral_constant<int, 2>{}); break;
        case 3: by_tail(std::integral_constant<int, 3>{}); break;
        case 4: by_tail(std::integral_constant<int, 4>{}); break;
        default: return hipErrorInvalidValue;
    }
    return dlk::launch_status();
}

// Forward pass with a handful of OUTPUT channels and 256 input channels (the logits layer):
//   D[m][k] = sum_{c < 256} A[m][c] * B[k][c],  k < KK <= THIN_MAX, dense rows of KK values.
// A bandwidth-bound sweep over A.  A lane owns one 16-byte chunk (8 channels) of a pixel and keeps the
// matching filter values in registers; the 32 lanes of a pixel (half a wavefront) add their partial dot
// products with four DPP row shifts and a row broadcast, lanes 31 and 63 park the two pixels' sums in LDS
// and the lanes that will store them read them back.  A wavefront works through runs of 16 consecutive pixels
// (8 trips of 1 KB), the next run's loads issued before the current run's arithmetic, and writes a run's
// 16 * KK results as one contiguous row of 2-byte stores.  Every sum is formed in a fixed order.
constexpr int TC_CIN = 256, TC_RUN = 16;

template <class T, int KK, bool TAIL>
__global__ __launch_bounds__(256) void thin_cols_kernel(const IgemmArgs p)
{
    __shared__ float sy[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane & 31, half = lane >> 5;
    float w[KK][8];
#pragma unroll
    for (int k = 0; k < KK; ++k) {
        const u32x4_t wv = *reinterpret_cast<const u32x4_t *>(p.B + (size_t)k * TC_CIN + g * 8);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            w[k][2 * d] = T::to_float((uint16_t)(wv[d] & 0xffffu));
            w[k][2 * d + 1] = T::to_float((uint16_t)(wv[d] >> 16));
        }
    }
    const int64_t M = (int64_t)p.NB * p.OH * p.OW;
    const int64_t runs = (M + TC_RUN - 1) / TC_RUN, stride = (int64_t)gridDim.x * 4;
    auto load_run = [&](u32x4_t (&v)[8], int64_t run) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            int64_t m = run * TC_RUN + 2 * t + half;             // past the end (last run only): re-read the last pixel,
            m = m < M ? m : M - 1;                               // its results are not stored
            v[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p.A + m * TC_CIN + g * 8));
        }
    };
    auto shr = [](float t, auto ctrl) {      // row_shr:n reads lane - n of the same row of 16 lanes, zero outside it
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    // the arithmetic of one run whose chunks are in `x`
    auto process = [&](const u32x4_t (&x)[8], const int64_t run) {
        // the 8 * KK dot products of the run stage by stage (independent chains side by side, so that the
        // DPP steps do not wait on each other)
        float v[8][KK];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float xf[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                xf[2 * d] = T::to_float((uint16_t)(x[t][d] & 0xffffu));
                xf[2 * d + 1] = T::to_float((uint16_t)(x[t][d] >> 16));
            }
#pragma unroll
            for (int k = 0; k < KK; ++k) {
                float a = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) a += xf[e] * w[k][e];
                v[t][k] = a;
            }
        }
        auto all_chains = [&](auto ctrl) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int k = 0; k < KK; ++k) v[t][k] += shr(v[t][k], ctrl);
        };
        all_chains(std::integral_constant<int, 0x111>{});
        all_chains(std::integral_constant<int, 0x112>{});
        all_chains(std::integral_constant<int, 0x114>{});
        all_chains(std::integral_constant<int, 0x118>{});        // lane 15 of every row of 16: the row's sum
        // row_bcast:15 into rows 1 and 3: lanes 31 and 63 then hold the sums of the trip's two pixels;
        // they park them in the wavefront's LDS row, from where lane i picks up result i of the run
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int k = 0; k < KK; ++k)
                v[t][k] += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[t][k]), 0x142, 0xa, 0xf, false));
        if (g == 31) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int k = 0; k < KK; ++k) sy[wave][(2 * t + half) * KK + k] = v[t][k];
        }
        const float outv = sy[wave][lane];               // same wavefront: LDS operations complete in order
        const int64_t first = run * TC_RUN * KK;             // flat index of the run's first result
        if (lane < TC_RUN * KK && first + lane < M * KK) {
            float r = outv;
            if constexpr (TAIL) r = apply_tail(r, p.bias, p.relu, lane % KK);
            p.D[first + lane] = T::from_float(r);
        }
    };
    // two register sets take turns: the loads of the run after next are issued before a run's arithmetic
    int64_t run = (int64_t)blockIdx.x * 4 + wave;
    u32x4_t xa[8], xb[8];
    if (run < runs) load_run(xa, run);
    while (run < runs) {
        if (run + stride < runs) load_run(xb, run + stride);
        __builtin_amdgcn_sched_barrier(0);
        process(xa, run);
        __builtin_amdgcn_sched_barrier(0);
        run += stride;
        if (run >= runs) break;
        if (run + stride < runs) load_run(xa, run + stride);
        __builtin_amdgcn_sched_barrier(0);
        process(xb, run);
        __builtin_amdgcn_sched_barrier(0);
        run += stride;
    }
}

bool thin_cols_applicable(const IgemmArgs &a)
{
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW &&
                       a.IH == a.OH && a.IW == a.OW && a.ooh == 0 && a.oow == 0;
    return dense && a.TR == 1 && a.TS == 1 && a.th0 == 0 && a.tw0 == 0 && a.Cin == TC_CIN && a.Nout >= 1 &&
           a.Nout <= THIN_MAX && a.ldd == a.Nout && !a.resid && !a.b_transposed;
}

hipError_t launch_thin_cols(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    if (M <= 0) return hipSuccess;
    const int64_t runs = (M + TC_RUN - 1) / TC_RUN;
    const int64_t want = (runs + 3) / 4;                  // one run per wavefront at least
    const dim3 grid((unsigned)(want < 2048 ? want : 2048)), block(256);
    const bool tail = a.bias || a.relu;
    auto go = [&](auto kk, auto has_tail) {
        constexpr int KK = decltype(kk)::value;
        constexpr bool TAIL = decltype(has_tail)::value;
        if (is_bf16) DLK_LAUNCH("thin_cols_kernel", (thin_cols_kernel<BF16, KK, TAIL>), grid, block, 0, stream, a);
        else DLK_LAUNCH("thin_cols_kernel", (thin_cols_kernel<F16, KK, TAIL>), grid, block, 0, stream, a);
    };
    auto by_tail = [&](auto kk) {
        if (tail) go(kk, std::true_type{});
        else go(kk, std::false_type{});
    };
    switch (a.Nout) {
        case 1: by_tail(std::integral_constant<int, 1>{}); break;
        case 2: by_tail(std::integral_constant<int, 2>{}); break;
        case 3: by_tail(std::integral_constant<int, 3>{}); break;
        case 4: by_tail(std::integral_constant<int, 4>{}); break;
        default: return hipErrorInvalidValue;
    }
    return dlk::launch_status();
}

// Filter gradient of a 1x1, stride-1, unpadded convolution with K <= THIN_MAX:
//   partial[b][k][c] = sum over workgroup b's pixels of dy[pix][k] * x[pix][c].
// A workgroup is (C/8 channel groups) x (256 / (C/8) pixel lanes); every thread
// keeps K x 8 running sums, the pixel lanes are then added in a fixed order.
// The workgroup's slice of dy is staged in LDS as fp32, 512 pixels at a time, so
// that the inner loop issues one 16-byte global load per pixel and nothing else.
// KK: the number of output channels (1..THIN_MAX) at compile time, so that the pixel loop is free of
// branches and the loads of four pixels are in flight before the first is used (with K read at run
// time every load was awaited right after its issue).  The sums of a thread run over its pixels in
// ascending order either way.
template <class T, int KK>
__global__ __launch_bounds__(256) void thin_wgrad_kernel(const WgradArgs p)
{
    constexpr int SUB = 512;                             // pixels of dy staged at a time
    __shared__ float red[256 * 8];                       // 8 sums per thread, reused for each k
    __shared__ __align__(16) float sdy[SUB * THIN_MAX];
    const int groups = p.C / 8;                          // <= 256
    const int lanes = 256 / groups;                      // pixel lanes per workgroup
    const int g = threadIdx.x % groups, pl = threadIdx.x / groups;
    const int npix = p.N * p.P * p.Q;
    const int pix_begin = blockIdx.x * p.chunk, pix_end = min(npix, pix_begin + p.chunk);
    float acc[KK][8];
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    auto add_pixel = [&](const u32x4_t xv, const int px) {
        const floatx4_t gd = *reinterpret_cast<const floatx4_t *>(sdy + px * THIN_MAX);   // one 16-byte broadcast read
        float xf[8];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            xf[2 * d] = T::to_float((uint16_t)(xv[d] & 0xffffu));
            xf[2 * d + 1] = T::to_float((uint16_t)(xv[d] >> 16));
        }
#pragma unroll
        for (int k = 0; k < KK; ++k)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[k][e] += gd[k] * xf[e];
    };
    for (int sub = pix_begin; sub < pix_end; sub += SUB) {
        const int sub_end = min(pix_end, sub + SUB);
        __syncthreads();                                 // the previous part of dy is no longer read
        for (int i = threadIdx.x; i < (sub_end - sub) * KK; i += 256) {
            const int px = i / KK, k = i - px * KK;
            sdy[px * THIN_MAX + k] = T::to_float(p.dy[(size_t)sub * KK + i]);
        }
        __syncthreads();
        if (pl < lanes) {
            const uint16_t *src = p.x + (size_t)(sub + pl) * p.C + g * 8;
            const size_t step = (size_t)lanes * p.C;
            // this lane's pixels of the part: n_l of them, `lanes` apart; groups of four are fetched one
            // group ahead of the arithmetic (the scheduling barriers keep the loads where they are written)
            const int n_l = (sub_end - sub - pl + lanes - 1) / lanes;
            const int ngroups = n_l >> 2;
            int px = pl;                                 // pixel within the part
            auto load4 = [&](u32x4_t (&v)[4], const uint16_t *q) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(q + i * step));
            };
            u32x4_t cur[4], nxt[4];
            if (ngroups > 0) load4(cur, src);
            for (int gi = 0; gi < ngroups; ++gi, px += 4 * lanes) {
                src += 4 * step;
                if (gi + 1 < ngroups) load4(nxt, src);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 4; ++i) add_pixel(cur[i], px + i * lanes);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 4; ++i) cur[i] = nxt[i];
            }
            for (; px < sub_end - sub; px += lanes, src += step)
                add_pixel(__builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src)), px);
        }
    }
    float *out = p.partial + (size_t)blockIdx.x * KK * p.C;
#pragma unroll
    for (int k = 0; k < KK; ++k) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) red[threadIdx.x * 8 + e] = (pl < lanes) ? acc[k][e] : 0.f;
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
    auto go = [&](auto kk) {
        constexpr int KK = decltype(kk)::value;
        if (is_bf16) DLK_LAUNCH("thin_wgrad_kernel", (thin_wgrad_kernel<BF16, KK>), grid, block, 0, stream, a);
        else DLK_LAUNCH("thin_wgrad_kernel", (thin_wgrad_kernel<F16, KK>), grid, block, 0, stream, a);
    };
    switch (a.K) {
        case 1: go(std::integral_constant<int, 1>{}); break;
        case 2: go(std::integral_constant<int, 2>{}); break;
        case 3: go(std::integral_constant<int, 3>{}); break;
        case 4: go(std::integral_constant<int, 4>{}); break;
        default: return hipErrorInvalidValue;
    }
    return dlk::launch_status();
}

}  // namespace dlk
