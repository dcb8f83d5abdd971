// Implicit-GEMM convolution engine for gfx950 (forward pass and, through a
// re-laid-out filter, the data gradient).
//
// GEMM view: M = N*OH*OW output pixels, N = output channels, reduction over
// (tap, input channel).  The im2col matrix is never materialised: each
// 16-byte load of 8 consecutive input channels computes its own source pixel
// from (output pixel, tap), which is where stride, padding and dilation
// enter.  Tiles are staged global -> registers -> LDS (two LDS buffers, one
// barrier per 32-deep step) and multiplied with v_mfma_f32_32x32x16.
#include "device_common.h"
#include "kernels.h"

namespace dlk {

template <int BM, int BN>
constexpr size_t igemm_lds_bytes() { return size_t(2) * (BM + BN) * LDS_PITCH * sizeof(uint16_t); }

// VEC: Cin % 8 == 0, so every 8-element slice of the reduction index stays
// inside one tap and is one aligned 16-byte load.  Otherwise elements are
// fetched one by one.
template <class T, int BM, int BN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(WM *WN * 64) void igemm_kernel(const IgemmArgs p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int ROWS_PER_PASS = NT / 4;          // 4 vectors of 8 elements per 32-deep row
    constexpr int PA = BM / ROWS_PER_PASS, PB = (BN + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
    constexpr bool B_PARTIAL = BN % ROWS_PER_PASS != 0;   // narrow filter tile: only rows < BN exist
    static_assert(BM % ROWS_PER_PASS == 0, "tile / thread-count mismatch");
    static_assert(TM >= 1 && TN >= 1, "wave tile too small");

    extern __shared__ __align__(16) uint16_t lds[];
    uint16_t *sA = lds;                                  // [2][BM][LDS_PITCH]
    uint16_t *sB = lds + 2 * BM * LDS_PITCH;             // [2][BN][LDS_PITCH]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int M = p.NB * p.OH * p.OW;
    const int Kred = p.TR * p.TS * p.Cin;
    const int tiles_n = (p.Nout + BN - 1) / BN;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    // ---- per-thread load coordinates: fixed rows, fixed 8-element column --
    const int vec = tid & 3, row0 = tid >> 2;
    int a_pix[PA], a_ih[PA], a_iw[PA];
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int m = m0 + row0 + i * ROWS_PER_PASS;
        if (m < M) {
            const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
            const int oh = rem / p.OW, ow = rem - oh * p.OW;
            a_pix[i] = n * p.IH * p.IW;
            a_ih[i] = oh * p.sh + p.th0;
            a_iw[i] = ow * p.sw + p.tw0;
        } else {
            a_pix[i] = 0;
            a_ih[i] = -(1 << 28);                        // fails every bounds test
            a_iw[i] = 0;
        }
    }
    // reduction index of this thread's slice: kk = (jr*TS + js)*Cin + c
    int kk = vec * 8;
    int c = kk % p.Cin, js = (kk / p.Cin) % p.TS, jr = (kk / p.Cin) / p.TS;

    u32x4_t ra[PA], rb[PB];
    auto load_tiles = [&]() {
        if constexpr (VEC) {
            const bool kin = kk < Kred;
            const int dh = jr * p.dth, dw = js * p.dtw;
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                const int ih = a_ih[i] + dh, iw = a_iw[i] + dw;
                const bool ok = kin && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (ok) v = *reinterpret_cast<const u32x4_t *>(p.A + (size_t)(a_pix[i] + ih * p.IW + iw) * p.Cin + c);
                ra[i] = v;
            }
#pragma unroll
            for (int i = 0; i < PB; ++i) {
                const int j = n0 + row0 + i * ROWS_PER_PASS;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (kin && j < p.Nout && (!B_PARTIAL || row0 + i * ROWS_PER_PASS < BN))
                    v = *reinterpret_cast<const u32x4_t *>(p.B + (size_t)j * Kred + kk);
                rb[i] = v;
            }
        } else {
            uint16_t ea[PA][8], eb[PB][8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k1 = kk + e;
                const bool kin = k1 < Kred;
                const int t = k1 / p.Cin, c1 = k1 - t * p.Cin;
                const int r1 = t / p.TS, s1 = t - r1 * p.TS;
#pragma unroll
                for (int i = 0; i < PA; ++i) {
                    const int ih = a_ih[i] + r1 * p.dth, iw = a_iw[i] + s1 * p.dtw;
                    const bool ok = kin && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                    ea[i][e] = ok ? p.A[(size_t)(a_pix[i] + ih * p.IW + iw) * p.Cin + c1] : (uint16_t)0;
                }
#pragma unroll
                for (int i = 0; i < PB; ++i) {
                    const int j = n0 + row0 + i * ROWS_PER_PASS;
                    const bool in_tile = !B_PARTIAL || row0 + i * ROWS_PER_PASS < BN;
                    eb[i][e] = (kin && j < p.Nout && in_tile) ? p.B[(size_t)j * Kred + k1] : (uint16_t)0;
                }
            }
#pragma unroll
            for (int i = 0; i < PA; ++i)
#pragma unroll
                for (int d = 0; d < 4; ++d) ra[i][d] = (uint32_t)ea[i][2 * d] | ((uint32_t)ea[i][2 * d + 1] << 16);
#pragma unroll
            for (int i = 0; i < PB; ++i)
#pragma unroll
                for (int d = 0; d < 4; ++d) rb[i][d] = (uint32_t)eb[i][2 * d] | ((uint32_t)eb[i][2 * d + 1] << 16);
        }
        // step this thread's slice to the next 32-deep block
        kk += BK;
        if constexpr (VEC) {
            c += BK;
            while (c >= p.Cin) {
                c -= p.Cin;
                if (++js == p.TS) { js = 0; ++jr; }
            }
        }
    };
    auto store_tiles = [&](int buf) {
        uint16_t *da = sA + buf * BM * LDS_PITCH + row0 * LDS_PITCH + vec * 8;
        uint16_t *db = sB + buf * BN * LDS_PITCH + row0 * LDS_PITCH + vec * 8;
#pragma unroll
        for (int i = 0; i < PA; ++i) *reinterpret_cast<u32x4_t *>(da + i * ROWS_PER_PASS * LDS_PITCH) = ra[i];
#pragma unroll
        for (int i = 0; i < PB; ++i)
            if (!B_PARTIAL || row0 + i * ROWS_PER_PASS < BN)
                *reinterpret_cast<u32x4_t *>(db + i * ROWS_PER_PASS * LDS_PITCH) = rb[i];
    };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = (Kred + BK - 1) / BK;
    if (nk > 0) {
        load_tiles();
        store_tiles(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < nk) load_tiles();
            mma_step<T, TM, TN>(sA + cur * BM * LDS_PITCH + wm * TM * 32 * LDS_PITCH,
                                sB + cur * BN * LDS_PITCH + wn * TN * 32 * LDS_PITCH, lane, acc);
            if (kt + 1 < nk) store_tiles(cur ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: round once, 32 lanes write 32 consecutive channels -----
    const bool dense = (p.osh == 1 && p.osw == 1 && p.FH == p.OH && p.FW == p.OW);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
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
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
                if (col < p.Nout) p.D[row_off + col] = T::from_float(acc[i][j][v]);
            }
        }
    }
}

template <class T, int BM, int BN, int WM, int WN, bool VEC>
static hipError_t launch_cfg(const IgemmArgs &a, hipStream_t stream)
{
    auto kern = igemm_kernel<T, BM, BN, WM, WN, VEC>;
    constexpr size_t lds = igemm_lds_bytes<BM, BN>();
    static bool attr_set = false;                       // raising the LDS limit is idempotent
    if (lds > 64 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    const int64_t tiles = ((M + BM - 1) / BM) * ((a.Nout + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(WM * WN * 64), lds, stream, a);
    return hipGetLastError();
}

template <class T>
static hipError_t dispatch(const IgemmArgs &a, hipStream_t stream)
{
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    if (a.Cin % 8 != 0) return launch_cfg<T, 128, 64, 2, 2, false>(a, stream);
    if (a.Nout <= 32) return launch_cfg<T, 128, 32, 4, 1, true>(a, stream);
    if (a.Nout <= 64) return launch_cfg<T, 128, 64, 2, 2, true>(a, stream);
    // wide outputs: the 256-row tile once there are enough of them to fill 256 CUs
    const int64_t big_tiles = ((M + 255) / 256) * ((a.Nout + 127) / 128);
    if (big_tiles >= 512) return launch_cfg<T, 256, 128, 2, 2, true>(a, stream);
    return launch_cfg<T, 128, 128, 2, 2, true>(a, stream);
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

hipError_t launch_filter_relayout(const FilterRelayoutArgs &a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.C * a.TR * a.TS * a.K;
    if (total <= 0) return hipSuccess;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(filter_relayout_kernel, dim3(blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace dlk
