// Filter-gradient kernel for dense 5x5 filters with unit stride, unit dilation
// and padding 2, at most 32 output channels, on large images (gfx950): the
// dense-block layers of a Tiramisu-style network (growth rate 32).
//
//   dw[k][r][s][c] = sum over pixels (n, y, x) of dy[n][y][x][k] * x[n][y+r-2][x+s-2][c]
//
// The general kernel treats every tap as its own GEMM column tile: 25 shifted
// activation tiles from L2 per block of pixels, and its smallest row tile (64)
// is half padding for 32 output channels.  Here a workgroup of five waves owns
// all k, one block of 32 input channels c and all 25 taps; wave s owns the
// five taps of column shift s (20 accumulator tiles of 16 x 16).  The
// workgroup walks down a strip of the image 32 pixels wide, one row per step:
//
//   step Y deposits row Y of x (36 pixels x 32 c: the strip plus two pixels
//   either side) and row Y+2 of dy (32 pixels x 32 k) in LDS; wave s reads its
//   shifted x fragments (2) and the new dy fragments (2) and issues
//       acc[r][s] += dy_row(Y - r + 2) * x_row(Y, shifted by s - 2)   for r = 0..4,
//   the dy fragments of the four previous rows staying in registers.
//
// That is 5 KB from L2 and 4 fragments per wave from LDS for 20 MFMAs of
// 16x16x32 per wave.  Both operands lie in memory with the reduction index
// (the pixel) as the slow axis; they are deposited pixel-major by
// `buffer_load_dwordx4 ... lds` and the fragments (8 pixels of one channel
// per lane) come from the LDS transpose read ds_read_b64_tr_b16.
//
// The image is cut into slices (a range of dy rows x a range of strips); a
// slice counts the products of ITS dy rows only (dy rows outside it read as
// zeros), with whatever x rows they meet.  Every (slice, channel block) writes
// fp32 partial sums, which the ordered reduce kernel adds.  Ring of five LDS
// slots (also the period of the dy register rotation), three steps in flight,
// one barrier per step; several workgroups share a compute unit.
#include <cstdlib>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

typedef short w5_s16x4_t __attribute__((ext_vector_type(4)));

template <class T>
__global__ __launch_bounds__(320) void wgrad5x5_kernel(const WgradStripArgs p)
{
    constexpr int NTAP = 5, PAD = 2;                     // five waves: one per column shift
    constexpr int KBLK = 32, CB = 32, PXB = 32;          // k per workgroup (all of them), c per workgroup, strip width
    constexpr int XROWS = 48;                            // x tile rows in LDS (36 used, three 16-row loads)
    constexpr int S = 5;                                 // ring slots = period of the dy register rotation
    constexpr int IN_FLIGHT = S - 2;                     // one load per wave per step
    constexpr int DY_ELEMS = PXB * KBLK, X_ELEMS = XROWS * CB, SLOT = DY_ELEMS + X_ELEMS;
    __shared__ __align__(16) uint16_t lds[S * SLOT];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which channel block of which slice ----------------------------------------
    const int tiles = (p.C + CB - 1) / CB;
    const int xcd = blockIdx.x % 8, slot_id = blockIdx.x / 8;
    const int tile = slot_id % tiles, slice = (slot_id / tiles) * 8 + xcd;
    if (slice >= p.slices) return;                       // uniform for the whole workgroup
    const int c0 = tile * CB;
    const int xblocks = (p.W + PXB - 1) / PXB;
    const int nxs = (xblocks + p.xs - 1) / p.xs, nrs = (p.H + p.rs - 1) / p.rs;
    const int img = slice / (nrs * nxs), rem = slice - img * (nrs * nxs);
    const int Y0 = (rem / nxs) * p.rs, Y1 = min(p.H, Y0 + p.rs);
    const int XB0 = (rem % nxs) * p.xs, XB1 = min(xblocks, XB0 + p.xs);

    const i32x4_t rsDY = make_rsrc_words(p.dy, (uint32_t)p.N * p.H * p.W * p.K * 2u);
    const i32x4_t rsX = make_rsrc_words(p.x, (uint32_t)p.N * p.H * p.W * p.C * 2u);

    // ---- what this lane fetches -------------------------------------------------
    // Waves 0, 1: a 16-pixel piece of the dy row each (64-byte pixel rows, 4 lanes per row).  The
    // 32-byte block b (16 channels) of pixel x sits at block b ^ ((x >> 2) & 1): the 8 pixel rows
    // a half-wave transpose read touches then fall on eight different bank ranges.
    const int d_pix = 16 * wave + (lane >> 2);
    const int d_blk = ((lane >> 1) & 1) ^ ((d_pix >> 2) & 1);
    const int d_ch = d_blk * 16 + (lane & 1) * 8;
    const bool d_ok = wave < 2 && d_ch < p.K;
    // Waves 2..4: the x tile, [16-channel block][48 rows][16 channels], so that 8 consecutive rows of
    // one block are 256 contiguous bytes whatever the shift; 16-byte position i = 64 * (wave - 2) +
    // lane holds block i / 96, row (i % 96) / 2, half i % 2 (rows 0..47, 36 used).
    const int x_pos = (wave - 2) * 64 + lane;
    const int x_row = (x_pos % (2 * XROWS)) >> 1, x_ch = c0 + (x_pos / (2 * XROWS)) * 16 + (x_pos & 1) * 8;
    const bool x_ok = wave >= 2 && x_row < PXB + 2 * PAD && x_ch < p.C;

    // load cursor (wave-uniform): strip ld_xb, x row ld_Y in [Y0 - 2, Y1 + 2)
    int ld_xb = XB0, ld_Y = Y0 - PAD;
    auto issue = [&](int slot) {
        const uint32_t dst = lds_addr(lds) + slot * (SLOT * 2);
        const bool live = ld_xb < XB1;                   // past the last strip: zeros
        if (wave < 2) {                                  // dy row ld_Y + 2, if it is one of the slice's
            const int y = ld_Y + PAD, px = ld_xb * PXB + d_pix;
            const bool ok = live && d_ok && y >= Y0 && y < Y1 && px < p.W;
            const uint32_t off = ok ? (uint32_t)(((img * p.H + y) * p.W + px) * p.K + d_ch) * 2u : OOB_OFFSET;
            dma_load_16B(rsDY, dst + wave * 1024, off);
        } else {                                         // x row ld_Y
            const int px = ld_xb * PXB - PAD + x_row;
            const bool ok = live && x_ok && (unsigned)ld_Y < (unsigned)p.H && (unsigned)px < (unsigned)p.W;
            const uint32_t off = ok ? (uint32_t)(((img * p.H + ld_Y) * p.W + px) * p.C + x_ch) * 2u : OOB_OFFSET;
            dma_load_16B(rsX, dst + DY_ELEMS * 2 + (wave - 2) * 1024, off);
        }
        if (++ld_Y == Y1 + PAD) { ld_Y = Y0 - PAD; ++ld_xb; }
    };

    floatx4_t acc[NTAP][2][2];                           // [r][16-k block][16-c block], column shift s = wave
#pragma unroll
    for (int r = 0; r < NTAP; ++r)
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) acc[r][ab >> 1][ab & 1] = floatx4_t{0.f, 0.f, 0.f, 0.f};

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
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((w5_s16x4_t __attribute__((address_space(3))) *)ptr);
    };
    auto pack = [&](w5_s16x4_t lo, w5_s16x4_t hi) {
        u32x4_t r;
        const u32x2_t l2 = __builtin_bit_cast(u32x2_t, lo), h2 = __builtin_bit_cast(u32x2_t, hi);
        r[0] = l2[0]; r[1] = l2[1]; r[2] = h2[0]; r[3] = h2[1];
        return r;
    };
    // dy fragment: 16-channel block a, the 32 pixels of the row (pixel + 16 keeps the block position)
    auto read_dy = [&](const uint16_t *slot, int a) {
        const uint16_t *lo = slot + f_pix * KBLK + ((a ^ ((f_pix >> 2) & 1)) << 4) + f_sub;
        return pack(tr_read(lo), tr_read(lo + 16 * KBLK));
    };
    // x fragment: 16-channel block b, tile rows wave .. wave + 31 (tile row 0 is pixel x0 - 2)
    auto read_x = [&](const uint16_t *slot, int b) {
        const uint16_t *lo = slot + DY_ELEMS + b * (XROWS * 16) + (wave + f_pix) * 16 + f_sub;
        return pack(tr_read(lo), tr_read(lo + 16 * 16));
    };

    u32x4_t fa[NTAP][2], fb[2];                          // dy rows (rotating) x k blocks; this wave's x shift x c blocks
#pragma unroll
    for (int i = 0; i < NTAP; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) fa[i][j] = u32x4_t{0, 0, 0, 0};

    // Step k of a turn of five: ring slot k; the new dy row (tap row r = 0) goes into register set k,
    // the row fetched r steps ago (tap row r) is in set (k - r) mod 5.
    auto step = [&](auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        const uint16_t *slot = lds + k * SLOT;
        // this wave's load for the step has landed (three later ones may be in flight); after the barrier
        // everybody's has, and every wave is past its reads of the previous step's slot
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
        __builtin_amdgcn_sched_barrier(0);
        fa[k][0] = read_dy(slot, 0);
        fa[k][1] = read_dy(slot, 1);
        fb[0] = read_x(slot, 0);
        fb[1] = read_x(slot, 1);
        issue((k + S - 1) % S);
#pragma unroll
        for (int r = 0; r < NTAP; ++r)
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) {
                const int a = ab >> 1, b = ab & 1;
                T::mfma16_acc(acc[r][a][b], fa[(k - r + NTAP) % NTAP][a], fb[b]);
            }
    };

    // every strip takes rows + 4 steps (the last four bring zero dy rows, which also clears the register
    // sets for the next strip); the count is rounded up to whole turns (extra steps multiply zeros)
    const int nsteps = (XB1 - XB0) * (Y1 - Y0 + 2 * PAD);
    const int nturns = (nsteps + S - 1) / S;
#pragma unroll
    for (int k = 0; k < S - 1; ++k) issue(k);
    for (int turn = 0; turn < nturns; ++turn) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
        step(std::integral_constant<int, 4>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    mfma_acc_settle();

    // ---- partial sums: register v of lane l of block (a, b) holds k = 16a + 4*(l/16) + v, c = 16b + l%16 ----
    float *out = p.partial + (size_t)slice * p.K * (NTAP * NTAP) * p.C;
#pragma unroll
    for (int ab = 0; ab < 4; ++ab)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int a = ab >> 1, b = ab & 1;
            const int k = 16 * a + 4 * (lane >> 4) + v;
            const int c = c0 + 16 * b + (lane & 15);
            if (k >= p.K || c >= p.C) continue;
#pragma unroll
            for (int r = 0; r < NTAP; ++r) out[((size_t)k * (NTAP * NTAP) + r * NTAP + wave) * p.C + c] = acc[r][a][b][v];
        }
}

bool wgrad5x5_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw)
{
    static const int mode = tuning_knob("DLCONV_WGRAD5X5", 1); // tuning override: 0 = never
    return mode && R == 5 && S == 5 && sh == 1 && sw == 1 && ph == 2 && pw == 2 && dh == 1 && dw == 1 && C % 8 == 0 &&
           K % 8 == 0 && K <= 32 && (int64_t)N * H * W >= 20000 && W >= 32 && H >= 16;
}

// Rows and strips per slice: rounds of workgroups on the busiest XCD (32 CUs, two workgroups each),
// the length of a workgroup's run of steps, and the fp32 partial sums written and read back once per slice.
WgradStripPlan wgrad5x5_make_plan(int N, int H, int W, int C, int K)
{
    const int tiles = (C + 31) / 32;
    const int xblocks = (W + 31) / 32;
    const double outputs = (double)K * 25 * C;
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
            const int64_t rounds = (tiles * per_xcd + 63) / 64;
            const double steps = (double)xs * (rs + 4) + 10;
            const double cost = rounds * steps * 0.35 + slices * outputs * 8.0 / 4.0e6;
            if (cost < best_cost) {
                best_cost = cost;
                best = WgradStripPlan{(int)slices, rs, xs};
            }
        }
    }
    return best;
}

hipError_t launch_wgrad5x5(const WgradStripArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t tiles = (a.C + 31) / 32;
    const int64_t blocks = tiles * ((a.slices + 7) / 8) * 8;
    if (a.slices <= 0 || a.rs <= 0 || a.xs <= 0 || a.K > 32 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    // the slices must cover the image exactly as the kernel decodes them
    const int xblocks = (a.W + 31) / 32;
    if ((int64_t)a.N * ((a.H + a.rs - 1) / a.rs) * ((xblocks + a.xs - 1) / a.xs) != a.slices) return hipErrorInvalidValue;
    if (is_bf16) DLK_LAUNCH("wgrad5x5_kernel", wgrad5x5_kernel<BF16>, dim3((unsigned)blocks), dim3(320), 0, stream, a);
    else DLK_LAUNCH("wgrad5x5_kernel", wgrad5x5_kernel<F16>, dim3((unsigned)blocks), dim3(320), 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
