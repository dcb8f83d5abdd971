// Implicit-GEMM convolution engine for gfx950 (forward pass and, through a
// re-laid-out filter, the data gradient).
//
// GEMM view: M = N*OH*OW output pixels, N = output channels, reduction over
// (tap, input channel).  The im2col matrix is never materialised: every load
// computes its own source pixel from (output pixel, tap), which is where
// stride, padding and dilation enter.  This file holds the host-side choice of
// kernel and tile for one implicit GEMM, the element-wise kernel for channel
// counts that are not a multiple of 8, and the filter re-layout for data
// gradients that cannot read the filter in place.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

// ===========================================================================
// Scalar kernel: any channel count; elements are fetched one by one.  Used
// only when Cin is not a multiple of 8.
// ===========================================================================
template <class T>
__global__ __launch_bounds__(256) void igemm_scalar_kernel(const IgemmArgs p)
{
    constexpr int BM = 128, BN = 64, WN = 2, TM = 2, TN = 1, RPP = 64, PA = 2, PB = 1;
    __shared__ __align__(16) uint16_t sA[BM * LDS_PITCH];
    __shared__ __align__(16) uint16_t sB[BN * LDS_PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int M = p.NB * p.OH * p.OW;
    const int Kred = p.TR * p.TS * p.Cin;
    const int tiles_n = (p.Nout + BN - 1) / BN;
    const int m0 = (blockIdx.x / tiles_n) * BM, n0 = (blockIdx.x % tiles_n) * BN;

    const int vec = tid & 3, row0 = tid >> 2;
    int a_pix[PA], a_ih[PA], a_iw[PA];
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int m = m0 + row0 + i * RPP;
        if (m < M) {
            const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
            const int oh = rem / p.OW, ow = rem - oh * p.OW;
            a_pix[i] = n * p.IH * p.IW;
            a_ih[i] = oh * p.sh + p.th0;
            a_iw[i] = ow * p.sw + p.tw0;
        } else {
            a_pix[i] = 0;
            a_ih[i] = -(1 << 28);
            a_iw[i] = 0;
        }
    }

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][0][v] = 0.f;

    const int nk = (Kred + BK - 1) / BK;
    for (int kt = 0; kt < nk; ++kt) {
        uint16_t ea[PA][8], eb[PB][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k1 = kt * BK + vec * 8 + e;
            const bool kin = k1 < Kred;
            const int t = k1 / p.Cin, c1 = k1 - t * p.Cin;
            const int r1 = t / p.TS, s1 = t - r1 * p.TS;
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                const int ih = a_ih[i] + r1 * p.dth, iw = a_iw[i] + s1 * p.dtw;
                const bool ok = kin && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                ea[i][e] = ok ? p.A[(size_t)(a_pix[i] + ih * p.IW + iw) * p.Cin + c1] : (uint16_t)0;
            }
            const int j = n0 + row0;
            eb[0][e] = (kin && j < p.Nout) ? p.B[(size_t)j * Kred + k1] : (uint16_t)0;
        }
        __syncthreads();                                 // previous step's fragment reads are done
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            u32x4_t v;
#pragma unroll
            for (int d = 0; d < 4; ++d) v[d] = (uint32_t)ea[i][2 * d] | ((uint32_t)ea[i][2 * d + 1] << 16);
            *reinterpret_cast<u32x4_t *>(sA + (row0 + i * RPP) * LDS_PITCH + vec * 8) = v;
        }
        {
            u32x4_t v;
#pragma unroll
            for (int d = 0; d < 4; ++d) v[d] = (uint32_t)eb[0][2 * d] | ((uint32_t)eb[0][2 * d + 1] << 16);
            *reinterpret_cast<u32x4_t *>(sB + row0 * LDS_PITCH + vec * 8) = v;
        }
        __syncthreads();
        mma_step<T, TM, TN, BK>(sA + wm * TM * 32 * LDS_PITCH, sB + wn * TN * 32 * LDS_PITCH, lane, acc);
    }

    const bool dense = (p.osh == 1 && p.osw == 1 && p.FH == p.OH && p.FW == p.OW);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + (wm * TM + i) * 32 + acc_row(v, lane);
            if (m >= M) continue;
            size_t row_off;
            if (dense) {
                row_off = (size_t)m * p.ldd;
            } else {
                const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
                const int oh = rem / p.OW, ow = rem - oh * p.OW;
                row_off = ((size_t)(n * p.FH + oh * p.osh + p.ooh) * p.FW + ow * p.osw + p.oow) * p.ldd;
            }
            const int col = n0 + wn * 32 + (lane & 31);
            if (col < p.Nout) {
                const float r = p.resid ? T::to_float(p.resid[row_off + col]) : 0.f;
                p.D[row_off + col] = T::from_float(apply_tail(acc[i][0][v] + r, p.bias, p.relu, col));
            }
        }
}

// ===========================================================================
// Host side: tile selection and launch
// ===========================================================================
// Tuning override: DLCONV_IGEMM_CFG=<n> forces tile configuration n for every
// vector-path launch (used by the tile sweeps; unset in normal use).
static int forced_cfg()
{
    static const int v = tuning_knob("DLCONV_IGEMM_CFG", -1);
    return v;
}

static bool choose_c_outer(const IgemmArgs &a)
{
    static const int force_order = tuning_knob("DLCONV_C_OUTER", -1);
    // channel-major order needs the tap mask to fit 64 bits and no chunk that is mostly padding
    const bool cm_ok = a.TR * a.TS <= 64;
    return cm_ok && (force_order >= 0 ? force_order != 0 : (a.Cin % 32 == 0 || a.Cin >= 128));
}

// Split of the reduction for GEMMs with few output pixels and a very long reduction (the
// ASPP 3x3 layers' forward pass: 6912 x 256 outputs, reduction 18432).  With tiles small enough
// to give every CU one, such a GEMM is bound by the L2 -> LDS traffic of its operand tiles
// (12 KB per 0.5 MFLOP step of a 128 x 64 tile: 1.5 GB, 12 TB/s).  Instead the 256 x 256 tile
// (a third of the traffic per FLOP) is used and ranges of channel chunks run side by side;
// an ordered reduce adds their fp32 partial sums.  Returns the number of ranges (1: no split)
// and the chunks per range.
static int choose_ksplits(const IgemmArgs &a, int *chunks_per_split)
{
    static const int mode = tuning_knob("DLCONV_KSPLIT", 1); // tuning override: 0 = never
    *chunks_per_split = 0;
    if (!mode || forced_cfg() >= 0 || a.Cin % 8 != 0 || !choose_c_outer(a)) return 1;
    const bool dense = a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW && a.ldd == a.Nout;
    if (!dense || a.Nout < 256 || a.Nout % 256 != 0) return 1;
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    const int64_t tiles = ((M + 255) / 256) * (a.Nout / 256);
    const int nchunks = (a.Cin + BK - 1) / BK;
    const int64_t steps = (int64_t)nchunks * a.TR * a.TS;
    if (steps < 256 || tiles > 64 || M * a.Nout > (4 << 20)) return 1;
    int64_t ks = 256 / tiles;                                 // one workgroup per CU
    if (ks > 8) ks = 8;
    if (ks > nchunks) ks = nchunks;
    if (ks < 2) return 1;
    const int cps = (int)((nchunks + ks - 1) / ks);
    *chunks_per_split = cps;
    return (nchunks + cps - 1) / cps;
}

size_t igemm_split_bytes(const IgemmArgs &a)
{
    int cps;
    const int ks = choose_ksplits(a, &cps);
    return ks > 1 ? (size_t)ks * a.NB * a.OH * a.OW * a.Nout * sizeof(float) : 0;
}

// Tile configuration of the direct-to-LDS engine for this GEMM (100 + its cfg), or the forced one.
static int choose_cfg(const IgemmArgs &a)
{
    int cfg = forced_cfg();
    if (cfg >= 0) return cfg;
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    // Largest tile that still yields enough workgroups for 256 CUs; tiles
    // wider than the output-channel count (rounded up to 64) are not considered.
    const int nmax = (a.Nout + 63) / 64 * 64;
    auto blocks = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((a.Nout + bn - 1) / bn); };
    if (nmax <= 32 || a.Nout <= 32) return 104;                     // 64 x 32
    if (nmax >= 256 && blocks(256, 256) >= 200) return 100;         // 256 x 256
    static const int min128 = tuning_knob("DLCONV_CFG128_MIN", 200); // tuning override: fewest 128 x 128 tiles that configuration is used for
    if (nmax >= 128 && blocks(128, 128) >= min128) return 102;      // 128 x 128
    if (blocks(128, 64) >= 200) return 103;                         // 128 x 64
    return 108;                                                     // 64 x 64
}

bool igemm_accepts_transposed_b(const IgemmArgs &a)
{
    static const int mode = tuning_knob("DLCONV_BT", 1); // tuning override: 0 = never
    return mode && a.Cin % 8 == 0 && a.Nout % 8 == 0 && a.Nout >= 32 && !(forced_cfg() < 0 && thin_rows_applicable(a)) && choose_cfg(a) >= 100 &&
           choose_c_outer(a);
}

template <class T>
static hipError_t dispatch(const IgemmArgs &a, hipStream_t stream)
{
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    if (forced_cfg() < 0 && thin_rows_applicable(a)) return launch_thin_rows(a, std::is_same<T, BF16>::value, stream);
    if (forced_cfg() < 0 && thin_cols_applicable(a)) return launch_thin_cols(a, std::is_same<T, BF16>::value, stream);
    if (a.Cin % 8 != 0) {
        const int64_t tiles = ((M + 127) / 128) * ((a.Nout + 63) / 64);
        if (tiles <= 0 || tiles > 0x7fffffff) return hipErrorInvalidValue;
        DLK_LAUNCH("igemm_scalar_kernel", igemm_scalar_kernel<T>, dim3((unsigned)tiles), dim3(256), 0, stream, a);
        return dlk::launch_status();
    }
    const int cfg = choose_cfg(a);
    if (cfg >= 100) {
        IgemmArgs b = a;
        b.c_outer = choose_c_outer(a);
        b.ksplits = 1;
        b.split_chunks = 0;
        if (a.part) {
            int cps;
            const int ks = choose_ksplits(a, &cps);
            if (ks > 1) {
                b.ksplits = ks;
                b.split_chunks = cps;
                hipError_t e = launch_igemm_dma(b, std::is_same<T, BF16>::value, 0, stream);      // 256 x 256 tiles
                if (e != hipSuccess) return e;
                return launch_splitk_reduce_tail(a.part, ks, M * a.Nout, a.D, std::is_same<T, BF16>::value ? 1 : 0, a.bias,
                                                 a.relu, a.Nout, a.resid, stream);
            }
        }
        // A ragged last column tile of the widest configuration (e.g. 304 = 256 + 48 output
        // channels) would run mostly empty: give the remainder to a narrower tile instead.
        const int rem = a.Nout % 256;
        if (cfg == 100 && a.Nout > 256 && rem != 0 && rem <= 128) {
            IgemmArgs lo = b, hi = b;
            lo.Nout = a.Nout - rem;
            hi.Nout = rem;
            if (a.b_transposed) hi.b_base = a.b_base + lo.Nout;
            else hi.B = a.B + (size_t)lo.Nout * a.TR * a.TS * a.Cin;
            hi.D = a.D + lo.Nout;
            if (a.bias) hi.bias = a.bias + lo.Nout;
            if (a.resid) hi.resid = a.resid + lo.Nout;
            hipError_t e = launch_igemm_dma(lo, std::is_same<T, BF16>::value, 0, stream);
            if (e != hipSuccess) return e;
            return launch_igemm_dma(hi, std::is_same<T, BF16>::value, rem <= 64 ? 3 : 2, stream);
        }
        return launch_igemm_dma(b, std::is_same<T, BF16>::value, cfg - 100, stream);
    }
    return hipErrorInvalidValue;                         // only the direct-to-LDS configurations (100 + n) exist
}

int igemm_batch_cfg(const IgemmArgs *a, int n)
{
    static const int mode = tuning_knob("DLCONV_BATCH", 1); // tuning override: 0 = one launch per GEMM
    if (!mode || n < 2 || n > IgemmBatch::MAX || forced_cfg() >= 0) return -1;
    // Sharing a launch pays where the single launches are short (start-up and drain of a 10 us
    // kernel, four times over); long GEMMs run better one after the other (the 3x3 stride-2
    // layer that produces a 768 x 1152 x 256 tensor: 0.80 ms against 0.96 ms in one launch).
    double macs = 0;
    for (int i = 0; i < n; ++i) macs += (double)a[i].NB * a[i].OH * a[i].OW * a[i].Nout * a[i].Cin * a[i].TR * a[i].TS;
    if (macs > 1e10) return -1;
    int cfg = -1;
    for (int i = 0; i < n; ++i) {
        const IgemmArgs &g = a[i];
        if (g.Cin % 8 != 0 || thin_rows_applicable(g) || thin_cols_applicable(g) || !choose_c_outer(g) || g.b_transposed != a[0].b_transposed) return -1;
        int cps;
        if (choose_ksplits(g, &cps) > 1) return -1;
        const int c = choose_cfg(g);
        const int rem = g.Nout % 256;
        if (c < 100 || (c == 100 && g.Nout > 256 && rem != 0 && rem <= 128)) return -1;    // that case is cut into two launches
        if (cfg >= 0 && c != cfg) return -1;
        cfg = c;
    }
    return cfg - 100;
}

hipError_t launch_igemm_batch(const IgemmBatch &b, bool is_bf16, hipStream_t stream)
{
    const int cfg = igemm_batch_cfg(b.a, b.n);
    if (cfg < 0) return hipErrorInvalidValue;
    IgemmBatch c = b;
    for (int i = 0; i < c.n; ++i) {
        c.a[i].c_outer = 1;
        c.a[i].ksplits = 1;
        c.a[i].split_chunks = 0;
        c.a[i].part = nullptr;
    }
    return launch_igemm_dma_batch(c, is_bf16, cfg, stream);
}

hipError_t launch_igemm(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    return is_bf16 ? dispatch<BF16>(a, stream) : dispatch<F16>(a, stream);
}

// ---- filter re-layout for the data gradient -------------------------------
__global__ void filter_relayout_kernel(const FilterRelayoutArgs p)
{
    const int64_t total = (int64_t)p.C * p.TR * p.TS * p.K;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int64_t t = i;
        const int k = (int)(t % p.K); t /= p.K;
        const int js = (int)(t % p.TS); t /= p.TS;
        const int jr = (int)(t % p.TR); t /= p.TR;
        const int c = (int)t;
        const int r = p.r0 + jr * p.rstep, s = p.s0 + js * p.sstep;
        p.wt[i] = p.w[(((int64_t)k * p.R + r) * p.S + s) * p.C + c];
    }
}

// Zero fill of the input-gradient pixels that no filter tap reaches (a 1x1 filter with stride 2 reads one pixel
// in four): pixel (h, w) belongs to stride-parity class (h % sh) * sw + (w % sw); the classes whose bit is set in
// `mask` are cleared, 16 bytes per thread, all of them in one sweep over the tensor (C % 8 == 0).
__global__ __launch_bounds__(256) void zero_classes_kernel(uint16_t *__restrict__ dx, int64_t pieces, int H, int W, int C8, int sh,
                                                           int sw, uint64_t mask)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (int64_t)gridDim.x * 256) {
        const int64_t pix = i / C8;
        const int w = (int)(pix % W), h = (int)((pix / W) % H);
        if ((mask >> ((h % sh) * sw + (w % sw))) & 1) *reinterpret_cast<u32x4_t *>(dx + i * 8) = u32x4_t{0, 0, 0, 0};
    }
}

hipError_t launch_zero_classes(uint16_t *dx, int N, int H, int W, int C, int sh, int sw, uint64_t mask, hipStream_t stream)
{
    if (C % 8 != 0 || sh < 1 || sw < 1 || sh * sw > 64) return hipErrorInvalidValue;
    const int64_t pieces = (int64_t)N * H * W * (C / 8);
    if (pieces <= 0 || mask == 0) return hipSuccess;
    const int64_t want = (pieces + 256 * 8 - 1) / (256 * 8);          // about eight pieces per thread
    const dim3 grid((unsigned)(want < 65535 ? want : 65535)), block(256);
    DLK_LAUNCH("zero_classes_kernel", zero_classes_kernel, grid, block, 0, stream, dx, pieces, H, W, C / 8, sh, sw, mask);
    return dlk::launch_status();
}

hipError_t launch_filter_relayout(const FilterRelayoutArgs &a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.C * a.TR * a.TS * a.K;
    if (total <= 0) return hipSuccess;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    DLK_LAUNCH("filter_relayout_kernel", filter_relayout_kernel, dim3(blocks), dim3(256), 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
