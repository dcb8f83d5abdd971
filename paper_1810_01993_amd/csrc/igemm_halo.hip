// Implicit-GEMM convolution engine, halo-tile variant for stride-1 filters with
// several taps (gfx950): the forward pass and the data gradient of the 3x3
// layers.
//
// A workgroup owns a 16x16 patch of output pixels (GEMM M = 256) and 256 output
// channels.  For every 32-channel chunk of the reduction it deposits the patch
// *with its halo* ((16 + reach)^2 input pixels x 32 channels) in LDS once and
// then visits all taps, reading the MFMA fragments of tap (r, s) from the same
// LDS image at a shifted pixel offset.  Compared with fetching a separate
// 256 x 32 activation tile per tap, the activation traffic from L2 drops by
// taps * 256 / halo pixels (7x for a 3x3 filter), which is what limits the
// plain engine on the full-resolution layers.
//
// The filter is read from a re-laid-out copy [chunk][tap][output channel][32]
// (ragged chunk zero-filled), so that the 256 x 32 filter tile of a step is
// one contiguous 16 KB run spread evenly over the L2 channels.
//
// Loads are `buffer_load_dwordx4 ... lds` (out of range = zeros).  Filter
// tiles use a ring of four LDS slots, three steps in flight; the two halo
// buffers alternate per chunk, and the next chunk's halo is fetched in
// 1 KB pieces spread over the first steps of the current chunk.  Every step
// issues the same number of loads per wave (a piece that is not needed is an
// out-of-range load into a spare slot), so one constant wait count serves.
#include <cstdlib>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

constexpr int HALO_TH = 16, HALO_TW = 16;               // output patch
constexpr int HALO_BN = 256;

__device__ __forceinline__ int halo_swz(int row) { return (row >> 2) & 3; }

// AW: halo pieces (1 KB = 16 pixels x 32 channels) per wave; 8 waves => up to AW*128 halo pixels.
template <class T, int AW>
__global__ __launch_bounds__(512) void igemm_halo_kernel(const IgemmArgs p)
{
    constexpr int NW = 8, WN = 4, TM = 4, TN = 2;        // 2 x 4 waves, wave tile 128 x 64
    constexpr int BM = HALO_TH * HALO_TW, BN = HALO_BN;
    constexpr int BIW = BN / 16 / NW;                    // filter loads per wave per step
    constexpr int PER_STEP = BIW + 1;                    // + one halo piece (or its stand-in)
    constexpr int IN_FLIGHT = 2 * PER_STEP;
    constexpr int HALO_ROWS = AW * NW * 16;

    __shared__ __align__(16) uint16_t sH[2][HALO_ROWS * BK];          // halo images, alternating per chunk
    __shared__ __align__(16) uint16_t sB0[BN * BK], sB1[BN * BK], sB2[BN * BK], sB3[BN * BK];
    __shared__ __align__(16) uint16_t sSpare[NW * 16 * BK];           // target of stand-in loads

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int NT = p.TR * p.TS;
    const int nchunks = (p.Cin + BK - 1) / BK;
    // halo geometry: tap offsets th0 + jr*dth (dth may be negative)
    const int oy_min = min(p.th0, p.th0 + (p.TR - 1) * p.dth), ox_min = min(p.tw0, p.tw0 + (p.TS - 1) * p.dtw);
    const int HH = HALO_TH + (p.TR - 1) * abs(p.dth), HW = HALO_TW + (p.TS - 1) * abs(p.dtw);

    const int tiles_x = (p.OW + HALO_TW - 1) / HALO_TW, tiles_y = (p.OH + HALO_TH - 1) / HALO_TH;
    const int tiles_n = (p.Nout + BN - 1) / BN;
    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tn = tile % tiles_n; tile /= tiles_n;
    const int tx = tile % tiles_x; tile /= tiles_x;
    const int ty = tile % tiles_y;
    const int img = tile / tiles_y;
    const int y0 = ty * HALO_TH, x0 = tx * HALO_TW, n0 = tn * BN;

    const i32x4_t rsA = make_rsrc_words(p.A, (uint32_t)p.NB * p.IH * p.IW * p.Cin * 2u);
    const i32x4_t rsB = make_rsrc_words(p.B, (uint32_t)nchunks * NT * p.Nout * BK * 2u);

    // ---- what this lane fetches ---------------------------------------------
    const int lrow = lane >> 2;
    const int vec = (lane & 3) ^ halo_swz(lrow);
    const int lane_c = vec * 8;
    uint32_t h_off[AW];                                  // byte offset of (halo pixel, channel 8*vec), or out of range
#pragma unroll
    for (int a = 0; a < AW; ++a) {
        const int hp = (wave + a * NW) * 16 + lrow;
        const int hy = hp / HW, hx = hp - hy * HW;
        const int iy = y0 + oy_min + hy, ix = x0 + ox_min + hx;
        const bool ok = hy < HH && (unsigned)iy < (unsigned)p.IH && (unsigned)ix < (unsigned)p.IW;
        h_off[a] = ok ? (uint32_t)(((img * p.IH + iy) * p.IW + ix) * p.Cin + lane_c) * 2u : OOB_OFFSET;
    }
    uint32_t b_off[BIW];
#pragma unroll
    for (int i = 0; i < BIW; ++i) {
        const int j = n0 + (wave + i * NW) * 16 + lrow;
        b_off[i] = j < p.Nout ? (uint32_t)(j * BK + lane_c) * 2u : OOB_OFFSET;
    }

    // ---- cursors (all wave-uniform) -------------------------------------------
    int ld_t = 0, ld_chunk = 0;                          // step whose filter tile is fetched next
    int t = 0, jr = 0, js = 0, chunk = 0;                // step being multiplied

    auto issue_filter = [&](uint16_t *sb) {
        const uint32_t tile_b = (uint32_t)((ld_chunk * NT + ld_t) * p.Nout) * (BK * 2u);   // past the end: out of range
#pragma unroll
        for (int i = 0; i < BIW; ++i)
            dma_load_16B(rsB, lds_addr(sb) + (wave + i * NW) * 16 * BK * 2,
                         b_off[i] != OOB_OFFSET ? b_off[i] + tile_b : OOB_OFFSET);
        if (++ld_t == NT) { ld_t = 0; ++ld_chunk; }
    };
    // piece `a` of the halo image of chunk `ch` (zeros past the last chunk / in a ragged chunk)
    auto issue_halo_piece = [&](int a_sel, int ch) {
        uint32_t off = OOB_OFFSET;
        const int c0 = ch * BK;
#pragma unroll
        for (int a = 0; a < AW; ++a)
            if (a == a_sel && h_off[a] != OOB_OFFSET && lane_c < p.Cin - c0) off = h_off[a] + (uint32_t)c0 * 2u;
        dma_load_16B(rsA, lds_addr(&sH[ch & 1][0]) + (wave + a_sel * NW) * 16 * BK * 2, off);
    };
    auto issue_spare = [&]() { dma_load_16B(rsA, lds_addr(sSpare) + wave * 16 * BK * 2, OOB_OFFSET); };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- fragment addressing ---------------------------------------------------
    // filter: row (lane % 32) of a 32-row tile, 16-byte slice 2*ks + lane/32, swizzled by row
    const int frow = lane & 31;
    int foff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) foff[ks] = frow * BK + (((ks * 2 + (lane >> 5)) ^ halo_swz(frow)) << 3);
    // activations: output pixel (py, px) of the patch -> halo pixel py*HW + px (+ the tap's shift)
    int hb[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int ml = (wm * TM + i) * 32 + frow;
        hb[i] = (ml / HALO_TW) * HW + (ml % HALO_TW);
    }
    const int v0 = lane >> 5;                            // slice of ks = 0; ks = 1 is v0 + 2

    // The eight waves work in two groups of four (one wave of each group per
    // SIMD) that run half a step apart: while one group reads its fragments
    // from LDS and issues the next loads, the other keeps the matrix pipe busy,
    // and at the next barrier they swap.  Each step therefore has two barriers;
    // group 1 takes one extra barrier before the loop and group 0 one after it.
    u32x4_t fa[2][TM], fb[2][TN];
    auto read_frags = [&](const uint16_t *sb) {
        const int shift = (p.th0 + jr * p.dth - oy_min) * HW + (p.tw0 + js * p.dtw - ox_min);   // uniform
        const uint16_t *hal = &sH[chunk & 1][0];
        const uint16_t *wb = sb + wn * TN * 32 * BK;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int h = hb[i] + shift;
            const int e0 = h * BK + ((v0 ^ halo_swz(h)) << 3);       // element offset, ks = 0
            fa[0][i] = *reinterpret_cast<const u32x4_t *>(hal + e0);
            fa[1][i] = *reinterpret_cast<const u32x4_t *>(hal + (e0 ^ 16));   // slice v0 + 2: flips bit 1 of the slice
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[ks][j] = *reinterpret_cast<const u32x4_t *>(wb + j * 32 * BK + foff[ks]);
    };
    auto multiply = [&]() {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = T::mfma(fa[s][i], fb[s][j], acc[i][j]);
    };
    auto advance = [&]() {
        ++t;
        if (++js == p.TS) { js = 0; ++jr; }
        if (t == NT) { t = 0; jr = 0; js = 0; ++chunk; }
    };
    // Barrier that opens a read phase: this wave's loads for the step about to be read have
    // landed (two later steps may be in flight) and its own LDS reads are complete.
    auto sync_loaded = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // Barrier between a wave's read phase and its multiply phase.  The other group opens its
    // read phase of the next step here, so this wave's loads for that step must have landed
    // too (it has issued one more step since its last wait, hence the same count), and its own LDS
    // reads must be complete, because after this barrier the other group refills the slot just read.
    auto sync_phase = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // One step of one wave: read this step's fragments, refill the ring slot freed by the
    // previous step with the filter tile three steps ahead, fetch one piece of the next
    // chunk's halo; then, one phase later, multiply.
    auto step = [&](uint16_t *sb_refill, const uint16_t *sb_cur) {
        sync_loaded();
        read_frags(sb_cur);
        issue_filter(sb_refill);
        if (t < AW) issue_halo_piece(t, chunk + 1);
        else issue_spare();
        advance();
        sync_phase();
        multiply();
    };

    const int nk = nchunks * NT;
    const int nturns = (nk + 3) / 4;                     // whole turns of the ring; extra steps multiply zeros
    // prologue: halo of chunk 0, then three filter tiles, each padded to PER_STEP loads
#pragma unroll
    for (int a = 0; a < AW; ++a) issue_halo_piece(a, 0);
    issue_filter(sB0); issue_spare();
    issue_filter(sB1); issue_spare();
    issue_filter(sB2); issue_spare();
    const bool late_group = wave >= NW / 2;              // waves 4..7: the second wave on each SIMD
    if (late_group) sync_loaded();
    for (int turn = 0; turn < nturns; ++turn) {
        step(sB3, sB0);
        step(sB0, sB1);
        step(sB1, sB2);
        step(sB2, sB3);
    }
    if (!late_group) sync_phase();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue ---------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ml = (wm * TM + i) * 32 + acc_row(v, lane);
            const int y = y0 + ml / HALO_TW, x = x0 + ml % HALO_TW;
            if (y >= p.OH || x >= p.OW) continue;
            const size_t row_off = ((size_t)(img * p.OH + y) * p.OW + x) * p.ldd;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
                if (col < p.Nout) {
                    const float r = p.resid ? T::to_float(p.resid[row_off + col]) : 0.f;
                    p.D[row_off + col] = T::from_float(apply_tail(acc[i][j][v] + r, p.bias, p.relu, col));
                }
            }
        }
    }
}

// ---- eligibility (shared by the workspace query and the launch) ---------------
static int halo_pieces_per_wave(const IgemmArgs &a)
{
    const int HH = HALO_TH + (a.TR - 1) * abs(a.dth), HW = HALO_TW + (a.TS - 1) * abs(a.dtw);
    const int rows = HH * HW;
    if (rows <= 3 * 128) return 3;
    if (rows <= 4 * 128) return 4;
    return 0;
}

static int halo_mode()
{
    static const int mode = tuning_knob("DLCONV_HALO", 1); // tuning override: 0 = never, 2 = general kernel only
    return mode;
}

static bool use_3x3(const IgemmArgs &a) { return halo_mode() == 1 && igemm_halo3x3_applicable(a); }
static bool use_narrow(const IgemmArgs &a) { return halo_mode() == 1 && igemm_narrow5x5_applicable(a); }
static bool use_wide(const IgemmArgs &a) { return halo_mode() == 1 && igemm_wide5x5_applicable(a); }

// Can a halo-tile kernel take all a.Nout columns?
static bool halo_takes(const IgemmArgs &a)
{
    if (!halo_mode() || a.Nout <= 0) return false;
    if (use_3x3(a)) return igemm_halo3x3_tiles(a) >= 200;
    const int NT = a.TR * a.TS;
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW;
    const int aw = halo_pieces_per_wave(a);
    if (!dense || a.Cin % 8 != 0 || aw == 0 || aw > NT - 2) return false;
    const int64_t tiles = (int64_t)a.NB * ((a.OH + HALO_TH - 1) / HALO_TH) * ((a.OW + HALO_TW - 1) / HALO_TW) *
                          ((a.Nout + HALO_BN - 1) / HALO_BN);
    return tiles >= 200;
}

// Leading output columns a halo-tile kernel takes (0 = none).  The 3x3 kernel takes any
// column count (it has a narrow variant for a short last tile); the general kernel leaves
// a trailing remainder that would fill less than about two thirds of its 256-wide tile
// to the plain engine.
int igemm_halo_columns(const IgemmArgs &a)
{
    if (!halo_mode()) return 0;
    if (use_narrow(a) || use_wide(a)) return a.Nout;     // 5x5 with at most 32 columns or 32 reduction channels: own kernels
    IgemmArgs h = a;
    if (!use_3x3(a)) {
        const int rem = a.Nout % HALO_BN;
        if (rem != 0 && rem < 160) h.Nout = a.Nout - rem;
    }
    return halo_takes(h) ? h.Nout : 0;
}

size_t igemm_blocked_filter_bytes(const IgemmArgs &a)
{
    return (size_t)((a.Cin + BK - 1) / BK) * a.TR * a.TS * a.Nout * BK * sizeof(uint16_t);
}

hipError_t launch_igemm_halo(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    if (use_narrow(a)) return launch_igemm_narrow5x5(a, is_bf16, stream);
    if (use_wide(a)) return launch_igemm_wide5x5(a, is_bf16, stream);
    const int64_t tiles = (int64_t)a.NB * ((a.OH + HALO_TH - 1) / HALO_TH) * ((a.OW + HALO_TW - 1) / HALO_TW) *
                          ((a.Nout + HALO_BN - 1) / HALO_BN);
    if (tiles <= 0 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    if (use_3x3(a)) return launch_igemm_halo3x3(a, is_bf16, stream);
    const dim3 grid((unsigned)tiles), block(512);
    const int aw = halo_pieces_per_wave(a);
    if (aw == 3) {
        if (is_bf16) DLK_LAUNCH("igemm_halo_kernel<3>", (igemm_halo_kernel<BF16, 3>), grid, block, 0, stream, a);
        else DLK_LAUNCH("igemm_halo_kernel<3>", (igemm_halo_kernel<F16, 3>), grid, block, 0, stream, a);
    } else if (aw == 4) {
        if (is_bf16) DLK_LAUNCH("igemm_halo_kernel<4>", (igemm_halo_kernel<BF16, 4>), grid, block, 0, stream, a);
        else DLK_LAUNCH("igemm_halo_kernel<4>", (igemm_halo_kernel<F16, 4>), grid, block, 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return dlk::launch_status();
}

// ---- filter re-layout into [chunk][tap][row][32] --------------------------------
// dst[((chunk*NT + jr*TS + js)*Nrows + j)*32 + e] = src[base + j*sj + jr*sr + js*ss + (chunk*32+e)*sc],
// zero where chunk*32 + e >= Cin.
__global__ void filter_block_kernel(const FilterBlockArgs p)
{
    const int64_t total = (int64_t)((p.Cin + BK - 1) / BK) * p.TR * p.TS * p.Nrows * BK;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = i;
        const int e = (int)(r % BK); r /= BK;
        const int j = (int)(r % p.Nrows); r /= p.Nrows;
        const int js = (int)(r % p.TS); r /= p.TS;
        const int jr = (int)(r % p.TR); r /= p.TR;
        const int c = (int)r * BK + e;
        p.dst[i] = c < p.Cin ? p.src[p.base + (int64_t)j * p.sj + (int64_t)jr * p.sr + (int64_t)js * p.ss + (int64_t)c * p.sc]
                             : (uint16_t)0;
    }
}

hipError_t launch_filter_block(const FilterBlockArgs &a, hipStream_t stream)
{
    const int64_t total = (int64_t)((a.Cin + BK - 1) / BK) * a.TR * a.TS * a.Nrows * BK;
    if (total <= 0) return hipSuccess;
    const int blocks = (int)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
    DLK_LAUNCH("filter_block_kernel", filter_block_kernel, dim3(blocks), dim3(256), 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
