// Filter-gradient kernel for dense 3x3 filters with unit stride, unit dilation
// and padding 1 on large images (gfx950): the full-resolution decoder layers.
//
//   dw[k][r][s][c] = sum over pixels (n, y, x) of dy[n][y][x][k] * x[n][y+r-1][x+s-1][c]
//
// The general kernel treats every tap as its own GEMM column tile and fetches a
// (shifted) activation tile and the same dy tile once per tap.  Here a
// workgroup owns 256 output channels k (32 per wave), ONE block of 32 input
// channels c and ALL NINE taps (9 accumulator tiles per wave), and walks down a
// strip of the image 32 pixels wide, one image row per step:
//
//   step Y deposits row Y of x (34 pixels x 32 c: the strip plus one pixel
//   either side) and row Y+1 of dy (32 pixels x 256 k) in LDS and issues
//       acc[r][s] += dy_row(Y - r + 1) * x_row(Y, shifted by s - 1)   for the 9 taps,
//   i.e. the x fragments of a row serve three taps with the dy fragments of
//   three consecutive rows, which stay in registers from step to step.
//
// Per step that is 18.2 KB from L2 and 8 fragments from LDS for 36 MFMAs of
// 16x16x32 per wave (the 32 pixels of the row are one reduction block; this
// MFMA shape draws less power per flop than 32x32x16, and the chip is
// power-limited), against 32 KB and 12 fragments in the general kernel.
// Both operands lie in memory with the reduction index (the pixel) as the slow
// axis; they are deposited pixel-major by `buffer_load_dwordx4 ... lds`, and the
// MFMA fragments (8 pixels of one channel per lane) come from the LDS transpose
// read ds_read_b64_tr_b16.
//
// The image is cut into slices (a range of rows x a range of strips); all
// channel-block tiles of a slice run on one XCD so that its rows of dy are
// fetched into that L2 once.  Every slice writes fp32 partial sums, which the
// ordered reduce kernel adds.  Steps alternate between two groups of four
// waves (read phase / multiply phase) as in the forward kernels; ring of six
// LDS slots, four steps in flight.
#include <cstdlib>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

typedef short w3_s16x4_t __attribute__((ext_vector_type(4)));

template <class T>
__global__ __launch_bounds__(512) void wgrad3x3_kernel(const WgradStripArgs p)
{
    constexpr int NW = 8;
    constexpr int KB = 256, CB = 32, PXB = 32;           // k per workgroup, c per workgroup, strip width
    constexpr int XROWS = 48;                            // x tile rows in LDS (34 used, three 16-row loads)
    constexpr int S = 6;                                 // ring slots
    constexpr int PER_STEP = 3;                          // loads per wave per step: 2 dy pieces + 1 x piece or stand-in
    constexpr int IN_FLIGHT = (S - 2) * PER_STEP;
    constexpr int DY_ELEMS = PXB * KB, X_ELEMS = XROWS * CB, SLOT = DY_ELEMS + X_ELEMS;

    __shared__ __align__(16) uint16_t lds[S * SLOT];
    __shared__ __align__(16) uint16_t sSpare[NW * 16 * CB];     // target of stand-in loads

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which tile of which slice ----------------------------------------------
    const int tiles_c = (p.C + CB - 1) / CB, tiles = tiles_c * ((p.K + KB - 1) / KB);
    const int xcd = blockIdx.x % 8, slot_id = blockIdx.x / 8;
    const int tile = slot_id % tiles, slice = (slot_id / tiles) * 8 + xcd;
    if (slice >= p.slices) return;                       // uniform for the whole workgroup
    const int c0 = (tile % tiles_c) * CB, k0 = (tile / tiles_c) * KB;
    const int xblocks = (p.W + PXB - 1) / PXB;
    const int nxs = (xblocks + p.xs - 1) / p.xs, nrs = (p.H + p.rs - 1) / p.rs;
    const int img = slice / (nrs * nxs), rem = slice - img * (nrs * nxs);
    const int Y0 = (rem / nxs) * p.rs, Y1 = min(p.H, Y0 + p.rs);
    const int XB0 = (rem % nxs) * p.xs, XB1 = min(xblocks, XB0 + p.xs);

    const i32x4_t rsDY = make_rsrc_words(p.dy, (uint32_t)p.N * p.H * p.W * p.K * 2u);
    const i32x4_t rsX = make_rsrc_words(p.x, (uint32_t)p.N * p.H * p.W * p.C * 2u);

    // ---- what this lane fetches -------------------------------------------------
    // dy tile: 512-byte pixel rows, 32 lanes per row; a load covers 2 pixel rows, wave w issues
    // loads w and w + 8 (pixels 2w + prow and 16 + 2w + prow).  Within a row the 32-byte block b
    // (16 channels) sits at block b ^ (pixel & 7): the 8 consecutive pixel rows of one block that
    // a half-wave transpose read touches then fall on eight different bank ranges.
    const int d_prow = lane >> 5, d_pchunk = lane & 31;
    const int d_pix = 2 * wave + d_prow;                 // pixel of the first load; the second is 16 further on
    const int d_blk = (d_pchunk >> 1) ^ (d_pix & 7);
    const int d_ch = k0 + ((d_blk << 1) | (d_pchunk & 1)) * 8;
    const bool d_ok = d_ch < p.K;
    // x tile: [16-channel block][48 rows][16 channels], so that 8 consecutive rows of one block
    // are 256 contiguous bytes whatever the shift; 16-byte position i = 64 * wave + lane holds
    // block i / 96, row (i % 96) / 2, half i % 2.  Waves 0..2 issue one load each (rows 0..47, 34 used).
    const int x_pos = wave * 64 + lane;
    const int x_row = (x_pos % (2 * XROWS)) >> 1, x_ch = c0 + (x_pos / (2 * XROWS)) * 16 + (x_pos & 1) * 8;
    const bool x_ok = wave < 3 && x_row < PXB + 2 && x_ch < p.C;

    // load cursor (wave-uniform): strip ld_xb, step row ld_Y in [Y0 - 2, Y1)
    int ld_xb = XB0, ld_Y = Y0 - 2;
    auto issue = [&](int slot) {
        const uint32_t dst = lds_addr(lds) + slot * (SLOT * 2);
        const bool live = ld_xb < XB1;                   // past the last strip: zeros
        {   // dy row ld_Y + 1
            const int y = ld_Y + 1;
            const bool row_ok = live && (unsigned)y < (unsigned)p.H;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int px = ld_xb * PXB + d_pix + 16 * i;
                const bool ok = row_ok && d_ok && px < p.W;
                const uint32_t off = ok ? (uint32_t)(((img * p.H + y) * p.W + px) * p.K + d_ch) * 2u : OOB_OFFSET;
                dma_load_16B(rsDY, dst + (wave + 8 * i) * 1024, off);
            }
        }
        {   // x row ld_Y (not during the two priming steps of a strip)
            const int px = ld_xb * PXB - 1 + x_row;
            const bool ok = live && x_ok && ld_Y >= Y0 && (unsigned)px < (unsigned)p.W;
            const uint32_t off = ok ? (uint32_t)(((img * p.H + ld_Y) * p.W + px) * p.C + x_ch) * 2u : OOB_OFFSET;
            const uint32_t xdst = wave < 3 ? dst + DY_ELEMS * 2 + wave * 1024 : lds_addr(sSpare) + wave * 1024;
            dma_load_16B(rsX, xdst, off);
        }
        if (++ld_Y == Y1) { ld_Y = Y0 - 2; ++ld_xb; }
    };

    floatx4_t acc[3][3][2][2];                           // [r][s][16-k block][16-c block]
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) acc[r][s][ab >> 1][ab & 1] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    // ---- fragment addressing for the transpose reads ------------------------------
    // lane = 16*g + q.  As a source it points at pixel 16*t + 4*g + q/4 (t = 0, 1: the two halves of
    // the group's 8 reduction elements; which pixel sits at which reduction position is free as
    // long as both operands agree) and channels 4*(q%4)..+3 of a 16-channel block; within a
    // 16-lane group lane i receives element i%4 of the words addressed by lanes 4j + i/4, i.e.
    // channel i of four pixels.
    const int g = lane >> 4, q = lane & 15;
    const int f_pix = 4 * g + (q >> 2);
    const int f_sub = 4 * (q & 3);
    auto tr_read = [&](const uint16_t *ptr) {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((w3_s16x4_t __attribute__((address_space(3))) *)ptr);
    };
    auto pack = [&](w3_s16x4_t lo, w3_s16x4_t hi) {
        u32x4_t r;
        const u32x2_t l2 = __builtin_bit_cast(u32x2_t, lo), h2 = __builtin_bit_cast(u32x2_t, hi);
        r[0] = l2[0]; r[1] = l2[1]; r[2] = h2[0]; r[3] = h2[1];
        return r;
    };
    // dy fragment: 16-channel block a of this wave's 32 channels, the 32 pixels of the row
    auto read_dy = [&](const uint16_t *slot, int a) {
        const int b = 2 * wave + a;
        const uint16_t *lo = slot + f_pix * KB + ((b ^ (f_pix & 7)) << 4) + f_sub;
        return pack(tr_read(lo), tr_read(lo + 16 * KB));
    };
    // x fragment: 16-channel block b, tile rows s .. s + 31 (tile row 0 is pixel x0 - 1)
    auto read_x = [&](const uint16_t *slot, int b, int s) {
        const uint16_t *lo = slot + DY_ELEMS + b * (XROWS * 16) + (s + f_pix) * 16 + f_sub;
        return pack(tr_read(lo), tr_read(lo + 16 * 16));
    };

    u32x4_t fa[3][2], fb[3][2];                          // dy rows (rotating) x k blocks; x shifts x c blocks
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) { fa[i][j] = u32x4_t{0, 0, 0, 0}; fb[i][j] = u32x4_t{0, 0, 0, 0}; }

    auto sync_loaded = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // The other group opens its read phase of the next step here, so this wave's loads for that
    // step must have landed too (it has issued one more step since its last wait: same count), and
    // its own LDS reads must be complete: after this barrier the other group refills the slot just read.
    auto sync_phase = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // Step k of a turn of six: ring slot k; the new dy row goes into register set k % 3, the rows
    // of the two previous steps are in sets (k+2) % 3 and (k+1) % 3.
    auto step = [&](auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        constexpr int n0 = k % 3, n1 = (k + 2) % 3, n2 = (k + 1) % 3;     // dy rows Y+1, Y, Y-1: taps r = 0, 1, 2
        const uint16_t *slot = lds + k * SLOT;
        sync_loaded();
        fa[n0][0] = read_dy(slot, 0);
        fa[n0][1] = read_dy(slot, 1);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            fb[s][0] = read_x(slot, 0, s);
            fb[s][1] = read_x(slot, 1, s);
        }
        issue((k + S - 1) % S);
        sync_phase();
#pragma unroll
        for (int ab = 0; ab < 4; ++ab)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int a = ab >> 1, b = ab & 1;
                T::mfma16_acc(acc[0][s][a][b], fa[n0][a], fb[s][b]);
                T::mfma16_acc(acc[1][s][a][b], fa[n1][a], fb[s][b]);
                T::mfma16_acc(acc[2][s][a][b], fa[n2][a], fb[s][b]);
            }
    };

    // steps: every strip takes rows + 2 steps (two priming steps fetch dy rows Y0-1 and Y0 while the x
    // tile is zero); the count is rounded up to whole turns of the ring (extra steps multiply zeros)
    const int nsteps = (XB1 - XB0) * (Y1 - Y0 + 2);
    const int nturns = (nsteps + S - 1) / S;
#pragma unroll
    for (int k = 0; k < S - 1; ++k) issue(k);
    const bool late_group = wave >= NW / 2;
    if (late_group) sync_loaded();
    for (int turn = 0; turn < nturns; ++turn) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
        step(std::integral_constant<int, 4>{});
        step(std::integral_constant<int, 5>{});
    }
    if (!late_group) sync_phase();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    mfma_acc_settle();

    // ---- partial sums: register v of lane l of block (a, b) holds k = 16a + 4*(l/16) + v, c = 16b + l%16 ----
    float *out = p.partial + (size_t)slice * p.K * 9 * p.C;
#pragma unroll
    for (int ab = 0; ab < 4; ++ab)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int a = ab >> 1, b = ab & 1;
            const int k = k0 + wave * 32 + 16 * a + 4 * (lane >> 4) + v;
            const int c = c0 + 16 * b + (lane & 15);
            if (k >= p.K || c >= p.C) continue;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) out[((size_t)k * 9 + r * 3 + s) * p.C + c] = acc[r][s][a][b][v];
        }
}

bool wgrad3x3_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw)
{
    static const int mode = tuning_knob("DLCONV_WGRAD3X3", 1); // tuning override: 0 = never
    return mode && R == 3 && S == 3 && sh == 1 && sw == 1 && ph == 1 && pw == 1 && dh == 1 && dw == 1 && C % 8 == 0 &&
           K % 8 == 0 && (int64_t)N * H * W >= 300000 && W >= 64 && H >= 16;
}

// Rows and strips per slice: what counts is how many rounds of workgroups the busiest XCD
// (32 CUs, one workgroup each) runs and how long a workgroup's run of steps is, plus the
// fp32 partial sums written and read back once per slice.
WgradStripPlan wgrad3x3_make_plan(int N, int H, int W, int C, int K)
{
    const int tiles = ((C + 31) / 32) * ((K + 255) / 256);
    const int xblocks = (W + 31) / 32;
    const double outputs = (double)K * 9 * C;
    WgradStripPlan best{0, 0, 0};
    double best_cost = 1e300;
    for (int nrs = 1; nrs <= H / 8 && nrs <= 64; ++nrs) {
        const int rs = (H + nrs - 1) / nrs;
        if ((H + rs - 1) / rs != nrs) continue;          // this row count does not give nrs slices
        for (int nxs = 1; nxs <= xblocks; ++nxs) {
            const int xs = (xblocks + nxs - 1) / nxs;
            if ((xblocks + xs - 1) / xs != nxs) continue;
            const int64_t slices = (int64_t)N * nrs * nxs;
            if (slices > 1024) break;
            const int64_t per_xcd = (slices + 7) / 8;
            const int64_t rounds = (tiles * per_xcd + 31) / 32;
            const double steps = (double)xs * (rs + 2) + 12;
            const double cost = rounds * steps * 0.55 + slices * outputs * 8.0 / 11.5e6;
            if (cost < best_cost) {
                best_cost = cost;
                best = WgradStripPlan{(int)slices, rs, xs};
            }
        }
    }
    return best;
}

hipError_t launch_wgrad3x3(const WgradStripArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t tiles = (int64_t)((a.C + 31) / 32) * ((a.K + 255) / 256);
    const int64_t blocks = tiles * ((a.slices + 7) / 8) * 8;
    if (a.slices <= 0 || a.rs <= 0 || a.xs <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    // the slices must cover the image exactly as the kernel decodes them
    const int xblocks = (a.W + 31) / 32;
    if ((int64_t)a.N * ((a.H + a.rs - 1) / a.rs) * ((xblocks + a.xs - 1) / a.xs) != a.slices) return hipErrorInvalidValue;
    if (is_bf16) DLK_LAUNCH("wgrad3x3_kernel", wgrad3x3_kernel<BF16>, dim3((unsigned)blocks), dim3(512), 0, stream, a);
    else DLK_LAUNCH("wgrad3x3_kernel", wgrad3x3_kernel<F16>, dim3((unsigned)blocks), dim3(512), 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
