// Filter-gradient kernel, direct-to-LDS variant (gfx950).
//
// GEMM view: rows = output channel k, columns j = (r*S + s)*C + c, reduction
// over the N*P*Q output pixels.  Both operands are channel-contiguous in
// memory (NHWC), i.e. the reduction index is their slow axis.  Tiles are
// therefore deposited in LDS as they lie in memory, [pixel][channel], by
// `buffer_load_dwordx4 ... lds` (zero for padding pixels, ragged edges and
// pixels past the end of the slice), and the MFMA fragments -- 8 consecutive
// pixels of one channel per lane -- are produced by the LDS transpose read
// ds_read_b64_tr_b16: within a group of 16 lanes, lane i receives element
// (i % 4) of the 64-bit words addressed by lanes 4j + i/4, j = 0..3.  Pointing
// lane s at pixel s/4, channels 4*(s%4)..+3 of a 4-pixel x 16-channel block
// hands lane i the 4 pixels of channel i.
//
// The pixel range is cut into `splits` slices; every slice writes an fp32
// partial tile and a second kernel adds the slices in a fixed order.
#include <cstdlib>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct PixCursor {            // (n, p, q) of one output pixel, advanced without division
    int n, p, q;
    __device__ __forceinline__ void init(int pix, int P, int Q) {
        n = pix / (P * Q);
        const int rem = pix - n * (P * Q);
        p = rem / Q;
        q = rem - p * Q;
    }
    __device__ __forceinline__ void advance(int by, int P, int Q) {
        q += by;
        while (q >= Q) {
            q -= Q;
            if (++p == P) { p = 0; ++n; }
        }
    }
};

// LDS image of a tile: row = pixel (BX channels = 2*BX bytes), and within a
// row the 32-byte block b (16 channels) sits at block b ^ (2 * (pixel & 3))
// (b ^ (pixel & 3) for rows of only four blocks).  Half a wave (the unit a
// 64-bit LDS read serves per cycle) touches four pixel rows x two adjacent
// blocks; rows are a multiple of the 256-byte bank width apart, and the rule
// puts those eight 32-byte pieces on eight different bank ranges.
__device__ __host__ constexpr int swz_shift(int BX) { return BX >= 128 ? 1 : 0; }
template <class T, int BM, int BN, int WM, int WN, int STAGES>
__global__ __launch_bounds__(WM *WN * 64) void wgrad_dma_kernel(const WgradArgs p)
{
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int LPR_A = BM / 8, LPR_B = BN / 8;          // lanes (16-byte chunks) per pixel row
    constexpr int PPI_A = 64 / LPR_A, PPI_B = 64 / LPR_B;  // pixel rows per load instruction
    constexpr int AIW = BK / PPI_A / NW, BIW = BK / PPI_B / NW;   // load instructions per wave per step
    static_assert(BM >= 64 && BN >= 64 && BM <= 512 && BN <= 512, "a row must be 4..32 chunks of 32 bytes");
    static_assert((BK / PPI_A) % NW == 0 && (BK / PPI_B) % NW == 0, "every wave must issue the same number of loads");
    static_assert(AIW >= 1 && BIW >= 1 && TM >= 1 && TN >= 1, "tile too small for this many waves");
    static_assert(STAGES == 3 || STAGES == 4, "ring of 3 or 4 LDS buffers");
    constexpr int IN_FLIGHT = (STAGES - 2) * (AIW + BIW);

    __shared__ __align__(16) uint16_t sA0[BK * BM], sA1[BK * BM], sA2[BK * BM], sA3[STAGES == 4 ? BK * BM : 8];
    __shared__ __align__(16) uint16_t sB0[BK * BN], sB1[BK * BN], sB2[BK * BN], sB3[STAGES == 4 ? BK * BN : 8];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int RSC = p.R * p.S * p.C;
    const int npix = p.N * p.P * p.Q;
    const int tiles_n = (RSC + BN - 1) / BN;
    const int tiles = tiles_n * ((p.K + BM - 1) / BM);
    // Workgroups are dealt to the 8 XCDs round-robin by id.  All tiles of one
    // pixel slice are given to the same XCD, back to back, so that the slice of
    // dy and x they all read is fetched into that XCD's L2 once.
    // With few slices (small images with large filters) that would leave XCDs idle: then
    // consecutive ids take consecutive tiles of a slice, i.e. every slice runs on all XCDs.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int tile = p.spread ? (int)(blockIdx.x % tiles) : slot % tiles;
    const int split = p.spread ? (int)(blockIdx.x / tiles) : (slot / tiles) * 8 + xcd;
    if (split >= p.splits) return;                         // uniform for the whole workgroup
    const int k0 = (tile / tiles_n) * BM, j0 = (tile % tiles_n) * BN;
    const int pix_begin = split * p.chunk;
    const int pix_end = min(npix, pix_begin + p.chunk);

    const i32x4_t rsA = make_rsrc_words(p.dy, (uint32_t)npix * p.K * 2u);
    const i32x4_t rsB = make_rsrc_words(p.x, (uint32_t)p.N * p.H * p.W * p.C * 2u);

    // ---- what this lane fetches --------------------------------------------
    // A (dy): instruction `inst` covers pixel rows inst*PPI_A .. +PPI_A-1 of the step
    const int a_prow = lane / LPR_A;                        // pixel row within an instruction
    const int a_pchunk = lane % LPR_A;                      // physical 16-byte chunk within the row
    // pixel & 3 is the same for all of this lane's instructions (see static_asserts on NW / PPI)
    const int a_pix3 = ((wave * PPI_A) + a_prow) & 3;
    const int a_ch = k0 + ((((a_pchunk >> 1) ^ (a_pix3 << swz_shift(BM))) << 1) | (a_pchunk & 1)) * 8;
    const bool a_ok = a_ch < p.K;

    const int b_prow = lane / LPR_B, b_pchunk = lane % LPR_B;
    const int b_pix3 = ((wave * PPI_B) + b_prow) & 3;
    const int b_col = j0 + ((((b_pchunk >> 1) ^ (b_pix3 << swz_shift(BN))) << 1) | (b_pchunk & 1)) * 8;
    const bool b_ok = b_col < RSC;
    const int b_tap = b_col / p.C, b_c = b_col - b_tap * p.C;
    const int b_r = b_tap / p.S, b_s = b_tap - b_r * p.S;
    const int b_dh = b_r * p.dh - p.ph, b_dw = b_s * p.dw - p.pw;
    static_assert((NW * PPI_A) % 4 == 0 && (NW * PPI_B) % 4 == 0, "swizzle must not depend on the instruction index");

    PixCursor cur[BIW];
#pragma unroll
    for (int i = 0; i < BIW; ++i) cur[i].init(pix_begin + (wave + i * NW) * PPI_B + b_prow, p.P, p.Q);
    int pix_base = pix_begin;                               // first pixel of the step being issued

    auto issue = [&](uint16_t *sa, uint16_t *sb) {
#pragma unroll
        for (int i = 0; i < AIW; ++i) {
            const int inst = wave + i * NW;
            const int pix = pix_base + inst * PPI_A + a_prow;
            const uint32_t off = (a_ok && pix < pix_end) ? (uint32_t)(pix * p.K + a_ch) * 2u : OOB_OFFSET;
            dma_load_16B(rsA, lds_addr(sa) + inst * 1024, off);
        }
#pragma unroll
        for (int i = 0; i < BIW; ++i) {
            const int inst = wave + i * NW;
            const int pix = pix_base + inst * PPI_B + b_prow;
            const int ih = cur[i].p * p.sh + b_dh, iw = cur[i].q * p.sw + b_dw;
            const bool ok = b_ok && pix < pix_end && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            const uint32_t off = ok ? (uint32_t)(((cur[i].n * p.H + ih) * p.W + iw) * p.C + b_c) * 2u : OOB_OFFSET;
            dma_load_16B(rsB, lds_addr(sb) + inst * 1024, off);
            cur[i].advance(BK, p.P, p.Q);
        }
        pix_base += BK;
    };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- fragment addressing for the transpose reads ------------------------
    // lane = 16*g + s.  As a source it points at pixel 8*(g>>1) + 4*t + s/4 (t = 0, 1: the two
    // halves of its 8-pixel slice) and channels 16*(g&1) + 4*(s%4)..+3 of a 32-channel MFMA tile.
    const int g = lane >> 4, s16 = lane & 15;
    const int f_pix = 8 * (g >> 1) + (s16 >> 2);            // + 4*t + 16*ks
    const int f_ch = 16 * (g & 1);                          // block-aligned part of the channel
    const int f_sub = 4 * (s16 & 3);                        // channel within the 16-channel block
    // element offset of (pixel, 32-channel tile `ct`, this lane) in a [BK][BX] tile
    auto frag_off = [&](int BX, int pix, int ch_tile0) {
        const int ch = ch_tile0 + f_ch;
        const int blk = (ch >> 4) ^ ((pix & 3) << swz_shift(BX));
        return pix * BX + blk * 16 + f_sub;
    };
    auto read_frag = [&](const uint16_t *tile, int BX, int ks, int ch_tile0) {
        const int p0 = 16 * ks + f_pix;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4_t __attribute__((address_space(3))) *)(tile + frag_off(BX, p0, ch_tile0)));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4_t __attribute__((address_space(3))) *)(tile + frag_off(BX, p0 + 4, ch_tile0)));
        u32x4_t r;
        const u32x2_t l2 = __builtin_bit_cast(u32x2_t, lo), h2 = __builtin_bit_cast(u32x2_t, hi);
        r[0] = l2[0]; r[1] = l2[1]; r[2] = h2[0]; r[3] = h2[1];
        return r;
    };
    auto mma = [&](const uint16_t *sa, const uint16_t *sb) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            u32x4_t a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = read_frag(sa, BM, ks, (wm * TM + i) * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = read_frag(sb, BN, ks, (wn * TN + j) * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = T::mfma(a[i], b[j], acc[i][j]);
        }
    };
    auto wait_and_sync = [&]() {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
    };

    // The step count is rounded up to a whole turn of the ring (the extra
    // steps load and multiply zeros) so that the unrolled loop has one exit.
    const int nk = pix_end > pix_begin ? (pix_end - pix_begin + BK - 1) / BK : 0;
    const int nturns = (nk + STAGES - 1) / STAGES;
    if (nk > 0) {
        issue(sA0, sB0);
        issue(sA1, sB1);
        if constexpr (STAGES == 4) issue(sA2, sB2);
        for (int turn = 0; turn < nturns; ++turn) {
            if constexpr (STAGES == 4) {
                wait_and_sync(); issue(sA3, sB3); mma(sA0, sB0);
                wait_and_sync(); issue(sA0, sB0); mma(sA1, sB1);
                wait_and_sync(); issue(sA1, sB1); mma(sA2, sB2);
                wait_and_sync(); issue(sA2, sB2); mma(sA3, sB3);
            } else {
                wait_and_sync(); issue(sA2, sB2); mma(sA0, sB0);
                wait_and_sync(); issue(sA0, sB0); mma(sA1, sB1);
                wait_and_sync(); issue(sA1, sB1); mma(sA2, sB2);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }

    float *out = p.partial + (size_t)split * p.K * RSC;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + (wm * TM + i) * 32 + acc_row(v, lane);
            if (k >= p.K) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = j0 + (wn * TN + j) * 32 + (lane & 31);
                if (col < RSC) out[(size_t)k * RSC + col] = acc[i][j][v];
            }
        }
}

template <class T, int BM, int BN, int WM, int WN, int STAGES>
static hipError_t launch_cfg(const WgradArgs &a, hipStream_t stream)
{
    const int RSC = a.R * a.S * a.C;
    const int64_t tiles = (int64_t)((a.K + BM - 1) / BM) * ((RSC + BN - 1) / BN);
    const int64_t split_groups = (a.splits + 7) / 8;        // each XCD takes every 8th slice
    const int64_t blocks = a.spread ? tiles * a.splits : tiles * split_groups * 8;
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    DLK_LAUNCH(kname("wgrad_dma_kernel", {BM, BN}), (wgrad_dma_kernel<T, BM, BN, WM, WN, STAGES>), dim3((unsigned)blocks), dim3(WM * WN * 64), 0,
                       stream, a);
    return dlk::launch_status();
}

WgradPlan wgrad_make_plan(int64_t npix, int K, int C, int RSC, bool thin_ok)
{
    static const int forced = tuning_knob("DLCONV_WGRAD_CFG", -2); // tuning override, unset in normal use
    WgradPlan pl{-1, 1, 32, 0};
    if (thin_ok && forced != -1) {
        // streaming kernel: one workgroup per slice of pixels, about eight slices per CU
        int64_t s = (npix + 255) / 256;
        if (s > 2048) s = 2048;
        if (s < 1) s = 1;
        pl.cfg = -2;
        pl.chunk = (int)((npix + s - 1) / s);
        pl.splits = (int)((npix + pl.chunk - 1) / pl.chunk);
        return pl;
    }
    const bool dma_ok = K % 8 == 0 && C % 8 == 0 && K >= 32 && RSC >= 64;
    if (!dma_ok || forced == -1 || forced > 3) {
        // register-transposing fallback kernel (128 x 128 tiles): about 1024 workgroups
        const int64_t tiles = (int64_t)((K + 127) / 128) * ((RSC + 127) / 128);
        int64_t s = (1024 + tiles - 1) / tiles;
        const int64_t max_by_len = (npix + 127) / 128;       // at least four 32-pixel steps per slice
        if (s > max_by_len) s = max_by_len;
        if (s > 512) s = 512;
        if (s < 1) s = 1;
        int64_t chunk = (npix + s - 1) / s;
        chunk = (chunk + 31) / 32 * 32;
        pl.chunk = (int)chunk;
        pl.splits = (int)((npix + chunk - 1) / chunk);
        return pl;
    }
    // Direct-to-LDS kernel: pick the tile shape and the number of pixel slices by a small
    // cost model.  The kernel gives all tiles of a slice to one XCD, so what counts is how
    // many rounds of workgroups the busiest XCD (32 CUs) has to run: a slice count that
    // leaves the last round almost empty costs a whole round.  Per round a workgroup spends
    // its reduction steps plus a fixed start-up; the fp32 partial tiles are written and read
    // back once per slice.  The constants are fitted to measured times on MI355X.
    struct Shape { int bm, bn, per_cu; double us_per_step; };
    static const Shape shapes[4] = {{256, 256, 1, 0.92}, {128, 128, 2, 0.55}, {64, 256, 2, 0.71}, {128, 256, 1, 0.88}};
    static const int forced_target = tuning_knob("DLCONV_WGRAD_TARGET", 0); // tuning override: workgroups wanted, unset in normal use
    const double outputs = (double)K * RSC;
    double best = 1e300;
    for (int cfg = 0; cfg < 4; ++cfg) {
        if (forced >= 0 && cfg != forced) continue;
        const Shape &sh = shapes[cfg];
        const int64_t tiles = (int64_t)((K + sh.bm - 1) / sh.bm) * ((RSC + sh.bn - 1) / sh.bn);
        const int64_t cap = 32 * sh.per_cu;                  // workgroups one XCD holds at a time
        for (int cand = 0; cand < 64 + 15; ++cand) {
            // 8, 16, ... 512 slices, the same number on every XCD, each slice on one XCD; or
            // 1 .. 15 slices whose tiles are dealt over all XCDs
            const bool spread = cand >= 64;
            int64_t s = spread ? cand - 63 : 8 * (cand + 1);
            if (forced_target > 0) s = (forced_target + tiles - 1) / tiles;
            if (s > 512) continue;
            if (s > 1 && s * 128 > npix) continue;           // at least four 32-pixel steps per slice
            int64_t chunk = (npix + s - 1) / s;
            chunk = (chunk + 31) / 32 * 32;
            const int64_t splits = (npix + chunk - 1) / chunk;
            const int64_t per_xcd = (splits + 7) / 8;
            const int64_t rounds = spread ? (tiles * splits + 8 * cap - 1) / (8 * cap) : (tiles * per_xcd + cap - 1) / cap;
            const double reduce_us = (splits > 1 ? splits * outputs * 8.0 : outputs * 6.0) / 11.5e6;
            const double est = 9.0 + rounds * (chunk / 32 + 7) * sh.us_per_step + reduce_us;
            if (est < best) {
                best = est;
                pl.cfg = cfg;
                pl.chunk = (int)chunk;
                pl.splits = (int)splits;
                pl.spread = spread ? 1 : 0;
            }
            if (forced_target > 0 && spread) break;
        }
    }
    return pl;
}

template <class T>
static hipError_t dispatch(const WgradArgs &a, int cfg, hipStream_t stream)
{
    switch (cfg) {
        case 0: return launch_cfg<T, 256, 256, 2, 4, 4>(a, stream);   // 8 waves, wave tile 128x64
        case 1: return launch_cfg<T, 128, 128, 2, 2, 4>(a, stream);   // 4 waves, wave tile 64x64
        case 2: return launch_cfg<T, 64, 256, 1, 4, 4>(a, stream);    // 4 waves, wave tile 64x64
        case 3: return launch_cfg<T, 128, 256, 2, 2, 4>(a, stream);   // 4 waves, wave tile 64x128
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_wgrad_dma(const WgradArgs &a, bool is_bf16, int cfg, hipStream_t stream)
{
    return is_bf16 ? dispatch<BF16>(a, cfg, stream) : dispatch<F16>(a, cfg, stream);
}

}  // namespace dlk
