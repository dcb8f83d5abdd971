// Halo-tile implicit-GEMM kernel specialised for dense 3x3 filters with unit
// stride and dilation (gfx950): the forward pass and the data gradient of the
// full-resolution decoder convolutions, where nearly all of the FLOPs are.
//
// A workgroup owns a 16-row x 32-column patch of output pixels (GEMM M = 512)
// and 128 output channels (variants: 160 and 64).  Compared with a square 256 x 256 tile the filter
// operand, which every workgroup has to re-fetch from L2 for every step, is
// half as wide, while the activation operand costs little because the patch is
// deposited in LDS once per 32-channel chunk together with its halo
// (18 x 34 pixels) and then serves all nine taps: 12.4 KB instead of 18.3 KB
// travel L2 -> LDS per step.
//
// The patch is 32 pixels wide so that one 32-row MFMA operand is exactly one
// patch row.  Moving a tap down by one row then means using the operand
// registers of the next row: a wave (4 patch rows x 64 channels) reads the six
// halo rows it needs once per column shift and uses each of them for up to
// three taps, which cuts the LDS -> register traffic of the activation operand
// in half.  Taps are therefore visited column shift by column shift, the row
// shift running fastest.
//
// Filter tiles come from the re-laid-out copy [chunk][tap][output channel][32]
// through a ring of six 8 KB LDS slots (five steps in flight); the halo of the
// next chunk is fetched in 1 KB pieces during the first five steps of the
// current one.  Every step issues the same number of loads per wave (one or two
// filter pieces and a halo piece, or their out-of-range stand-ins), so one
// constant wait count serves.
// The eight waves run as two groups half a step apart, as in the general
// halo-tile kernel.
#include <cstdlib>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

namespace {
constexpr int P3_PH = 16, P3_PW = 32, P3_BN = 128;
constexpr int P3_HH = P3_PH + 2, P3_HW = P3_PW + 2;
// Which 16-byte slice of a 64-byte row holds channel slice v: v ^ swz(row).  Lane l of a 16x16x32 MFMA operand
// reads slice l/16 of row l%16; with this rule a wavefront's ds_read_b128 of 16 consecutive rows takes its
// 4 cycles (256 B per cycle) at any alignment of the first row (measured with the LDS counters; the rule
// (row >> 2) & 3, right for 32-row operands, costs 8 cycles here).
__device__ __forceinline__ int p3_swz(int row) { return (row >> 1) & 3; }
}  // namespace

// NB: 16-channel blocks per wave (4: the 128-channel tile; 5: a 160-channel tile, for channel
// counts such as 304 that two of them cover with less waste; 2: a 64-channel tile for a narrow
// last column tile).  The launch covers output channels [col0, col0 + p.Nout) of a blocked filter
// copy that has bcols columns; p.D already points at column col0.
template <class T, int NB>
__global__ __launch_bounds__(512) void igemm_halo3x3_kernel(const IgemmArgs p, const int col0, const int bcols)
{
    constexpr int NW = 8, WN = 2, TM = 4;                // 4 x 2 waves, wave tile 4 patch rows x 16*NB channels
    constexpr int CH = NB * 16;                          // channels per wave
    constexpr int HW = P3_HW, HH = P3_HH, BN = WN * CH;
    constexpr int BPIECES = BN / 16;                     // 16-row filter pieces per step, dealt to the waves in turn
    constexpr int FPW = (BPIECES + NW - 1) / NW;         // filter loads per wave per step (stand-ins included)
    constexpr int NT = 9;
    constexpr int AW = 5;                                // halo pieces per wave: 5*8*16 = 640 >= 18*34 pixels
    constexpr int HALO_ROWS = AW * NW * 16;
    constexpr int S = 6;                                 // filter ring slots
    constexpr int PER_STEP = FPW + 1;
    constexpr int IN_FLIGHT = (S - 2) * PER_STEP;
    static_assert(AW <= NT - (S - 2), "a halo piece must have landed before its chunk starts");
    static_assert(HALO_ROWS >= HH * HW, "halo does not fit its pieces");
    static_assert(IN_FLIGHT < 64, "wait count field");

    // one array: two halo images (alternating per chunk), the filter ring, the target of stand-in
    // loads; the epilogue re-uses the front as staging space
    constexpr int H_ELEMS = HALO_ROWS * BK, B_ELEMS = BN * BK;
    __shared__ __align__(16) uint16_t lds[2 * H_ELEMS + S * B_ELEMS + NW * 16 * BK];
    uint16_t *const sH = lds, *const sB = lds + 2 * H_ELEMS, *const sSpare = sB + S * B_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int nchunks = (p.Cin + BK - 1) / BK;
    const bool flip_r = p.dth < 0, flip_s = p.dtw < 0;   // which tap a given shift belongs to
    const int oy_min = flip_r ? p.th0 - 2 : p.th0, ox_min = flip_s ? p.tw0 - 2 : p.tw0;

    const int tiles_x = (p.OW + P3_PW - 1) / P3_PW, tiles_y = (p.OH + P3_PH - 1) / P3_PH;
    const int tiles_n = (p.Nout + BN - 1) / BN;
    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tn = tile % tiles_n; tile /= tiles_n;
    const int tx = tile % tiles_x; tile /= tiles_x;
    const int ty = tile % tiles_y;
    const int img = tile / tiles_y;
    const int y0 = ty * P3_PH, x0 = tx * P3_PW, n0 = tn * BN;

    const i32x4_t rsA = make_rsrc_words(p.A, (uint32_t)p.NB * p.IH * p.IW * p.Cin * 2u);
    const i32x4_t rsB = make_rsrc_words(p.B, (uint32_t)nchunks * NT * bcols * BK * 2u);

    // ---- what this lane fetches ---------------------------------------------
    const int lrow = lane >> 2;
    const int vec = (lane & 3) ^ p3_swz(lrow);
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
    uint32_t b_off[FPW];                                 // this lane's filter rows: piece wave + f*NW of the tile
#pragma unroll
    for (int f = 0; f < FPW; ++f) {
        const int piece = wave + f * NW, bj = n0 + piece * 16 + lrow;
        b_off[f] = (piece < BPIECES && bj < p.Nout) ? (uint32_t)((col0 + bj) * BK + lane_c) * 2u : OOB_OFFSET;
    }

    // ---- cursors (all wave-uniform) -------------------------------------------
    int ld_rs = 0, ld_cs = 0, ld_chunk = 0;              // step whose filter tile is fetched next
    int cs = 0, chunk = 0;                               // step being multiplied (its row shift is compile-time)

    auto issue_filter = [&](int slot) {
        const int jr = flip_r ? 2 - ld_rs : ld_rs, js = flip_s ? 2 - ld_cs : ld_cs;
        const uint32_t tile_b = (uint32_t)((ld_chunk * NT + jr * 3 + js) * bcols) * (BK * 2u);   // past the end: out of range
        // a wave beyond the tile's pieces keeps the load count uniform with a stand-in (zeros into its spare area)
#pragma unroll
        for (int f = 0; f < FPW; ++f) {
            const int piece = wave + f * NW;
            const uint32_t dst = piece < BPIECES ? lds_addr(sB + slot * B_ELEMS) + piece * 16 * BK * 2 : lds_addr(sSpare) + wave * 16 * BK * 2;
            dma_load_16B(rsB, dst, b_off[f] != OOB_OFFSET ? b_off[f] + tile_b : OOB_OFFSET);
        }
        if (++ld_rs == 3) {
            ld_rs = 0;
            if (++ld_cs == 3) { ld_cs = 0; ++ld_chunk; }
        }
    };
    // piece `a_sel` of the halo image of chunk `ch` (zeros past the last chunk / in a ragged chunk)
    auto issue_halo_piece = [&](int a_sel, int ch) {
        uint32_t off = OOB_OFFSET;
        const int c0 = ch * BK;
#pragma unroll
        for (int a = 0; a < AW; ++a)
            if (a == a_sel && h_off[a] != OOB_OFFSET && lane_c < p.Cin - c0) off = h_off[a] + (uint32_t)c0 * 2u;
        dma_load_16B(rsA, lds_addr(sH + (ch & 1) * H_ELEMS) + (wave + a_sel * NW) * 16 * BK * 2, off);
    };
    auto issue_spare = [&]() { dma_load_16B(rsA, lds_addr(sSpare) + wave * 16 * BK * 2, OOB_OFFSET); };

    // The MFMA shape is 16x16x32: one instruction covers the whole 32-deep step for a 16-channel x
    // 16-pixel block.  (With operands distributed like real activations and filters the chip is
    // power-limited, and this shape sustains ~15 % more FLOP/s than 32x32x16 at the same power: a
    // register-resident loop reaches 1.65 against 1.43 PFLOP/s.)  acc[i][n][b]: patch row i,
    // 16-channel block n, pixel half b of the row.  The accumulators are pinned in place
    // (mfma16_acc): left to the register allocator, the 160-channel tile does not fit the
    // register file and the 128-channel tile only just.
    floatx4_t acc[TM][NB][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[i][n][b] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    // ---- fragment addressing ---------------------------------------------------
    // an operand tile is 16 rows (channels or pixels) x 32 reduction elements: lane l reads the
    // 16-byte slice l/16 of row l%16
    const int frow = lane & 15;
    const int fsl = lane >> 4;
    const int foff = frow * BK + ((fsl ^ p3_swz(frow)) << 3);        // filter; tile bases are multiples of 16 rows
    const int hbase = (wm * TM) * HW + frow;             // halo pixel of (first patch row of the wave, column frow), shift 0

    u32x4_t fa[TM + 2][2], fb[NB];
    // Halo row r (0..5) under the wave's four patch rows, at column shift cs_ of chunk ch_'s image;
    // [][b]: pixels 16*b .. +15 of the row.  The six rows of a column shift are not read in one
    // step: rows 2, 3 in the step of row shift 0, row 4 with row shift 1 and row 5 with row shift 2
    // (when they are first needed), and rows 0, 1 one step ahead, in the last step of the previous
    // column shift, whose products no longer use those registers.  That spreads the LDS reads
    // evenly over the steps (with the filter: 8, 6 and 10 instead of 16, 4 and 4).
    auto read_row = [&](int r, int cs_, int ch_) __attribute__((always_inline)) {
        const uint16_t *hal = sH + (ch_ & 1) * H_ELEMS;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int h = hbase + r * HW + cs_ + 16 * b;
            fa[r][b] = *reinterpret_cast<const u32x4_t *>(hal + h * BK + ((fsl ^ p3_swz(h)) << 3));
        }
    };
    auto read_filter = [&](int slot) {
        const uint16_t *wb = sB + slot * B_ELEMS + wn * CH * BK + foff;
#pragma unroll
        for (int n = 0; n < NB; ++n) fb[n] = *reinterpret_cast<const u32x4_t *>(wb + n * 16 * BK);
    };
    // Barrier that opens a read phase: this wave's loads for the step about to be read have
    // landed (S - 2 later steps may be in flight) and its own LDS reads are complete.
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
    // Step k of a turn of six: ring slot k, row shift k % 3.
    auto step = [&](auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        constexpr int u = k % 3;
        sync_loaded();
        if (u == 0) {
            if (chunk == 0 && cs == 0) { read_row(0, 0, 0); read_row(1, 0, 0); }   // nobody read them ahead
            read_row(2, cs, chunk);
            read_row(3, cs, chunk);
        } else if (u == 1) {
            read_row(4, cs, chunk);
        } else {
            read_row(5, cs, chunk);
            // The next column shift's rows 0, 1.  Across a chunk boundary they come from the next
            // chunk's image: its pieces that hold these rows (halo pixels < 512: pieces 0..3 of every
            // wave) were issued in steps 0..3 of this chunk, i.e. five or more steps ago: landed.
            const int ncs = cs == 2 ? 0 : cs + 1, nch = cs == 2 ? chunk + 1 : chunk;
            read_row(0, ncs, nch);
            read_row(1, ncs, nch);
        }
        read_filter(k);
        issue_filter((k + S - 1) % S);                   // the slot the previous step has finished with
        const int q = cs * 3 + u;                        // step within the chunk
        if (q < AW) issue_halo_piece(q, chunk + 1);
        else issue_spare();
        sync_phase();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int n = 0; n < NB; ++n)
#pragma unroll
                for (int b = 0; b < 2; ++b) T::mfma16_acc(acc[i][n][b], fb[n], fa[i + u][b]);   // rows = channels
        if (u == 2 && ++cs == 3) { cs = 0; ++chunk; }
    };

    const int nk = nchunks * NT;
    const int nturns = (nk + S - 1) / S;                 // whole turns of the ring; extra steps multiply zeros
    // prologue: halo of chunk 0, then five filter tiles, each padded to PER_STEP loads per wave
#pragma unroll
    for (int a = 0; a < AW; ++a) issue_halo_piece(a, 0);
#pragma unroll
    for (int k = 0; k < S - 1; ++k) { issue_filter(k); issue_spare(); }
    const bool late_group = wave >= NW / 2;              // waves 4..7: the second wave on each SIMD
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
    // every wave's loads (the trailing ones deposit zeros) and LDS reads are over before LDS is reused
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    mfma_acc_settle();

    // ---- epilogue ---------------------------------------------------------------
    // The filter rode in the first MFMA operand, so register v of lane l of a
    // 16x16 block holds channel 4*(l/16) + v of pixel l%16: four consecutive
    // channels per accumulator.  Each wave rounds its tile to 16 bits,
    // parks it in a private LDS area as [pixel][the wave's channels] (two patch
    // rows at a time) and writes it out as whole channel rows, 16 bytes per
    // lane.  Row pitch = channels + 16 bytes, i.e. an odd number of 16-byte
    // units: the 8-byte writes of 16 pixels x 2 channel quartets (a half-wave)
    // then fall on 32 different bank pairs, and the rows stay 16-byte aligned.
    constexpr int EP = CH + 8;                           // staging pitch in 16-bit elements
    static_assert(CH % 16 == 0 && (EP / 8) % 2 == 1, "staging pitch");
    constexpr int LPR = CH / 8;                          // lanes per pixel row when writing out
    static_assert(NW * 64 * EP <= 2 * H_ELEMS + S * B_ELEMS, "staging area must fit the tile buffers");
    uint16_t *stg = lds + wave * 64 * EP;
    const bool vec_ok = (p.ldd % 8 == 0) && (p.Nout % 8 == 0) && ((reinterpret_cast<uintptr_t>(p.D) & 15) == 0);
    const bool tail = p.bias != nullptr || p.relu != 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int n = 0; n < NB; ++n)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    floatx4_t c = acc[2 * h + ii][n][b];
                    if (tail) c = apply_tail4(c, p.bias, p.relu, n0 + wn * CH + n * 16 + 4 * (lane >> 4), p.Nout);
                    u32x2_t pk;
                    pk[0] = (uint32_t)T::from_float(c[0]) | ((uint32_t)T::from_float(c[1]) << 16);
                    pk[1] = (uint32_t)T::from_float(c[2]) | ((uint32_t)T::from_float(c[3]) << 16);
                    const int px = ii * 32 + b * 16 + (lane & 15), ch = n * 16 + 4 * (lane >> 4);
                    *reinterpret_cast<u32x2_t *>(stg + px * EP + ch) = pk;
                }
#pragma unroll
        for (int it = 0; it < LPR; ++it) {               // 64 pixels x LPR lanes, 64 lanes at a time
            const int item = it * 64 + lane;
            const int px = item / LPR, c8 = (item % LPR) * 8;
            const u32x4_t v4 = *reinterpret_cast<const u32x4_t *>(stg + px * EP + c8);
            const int y = y0 + wm * TM + 2 * h + (px >> 5), x = x0 + (px & 31);
            const int col = n0 + wn * CH + c8;
            if (y >= p.OH || x >= p.OW || col >= p.Nout) continue;
            uint16_t *dst = p.D + ((size_t)(img * p.OH + y) * p.OW + x) * p.ldd + col;
            if (vec_ok) {
                *reinterpret_cast<u32x4_t *>(dst) = v4;
            } else {
                const uint32_t w4[4] = {v4[0], v4[1], v4[2], v4[3]};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (col + e < p.Nout) dst[e] = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

bool igemm_halo3x3_applicable(const IgemmArgs &a)
{
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW;
    return dense && a.TR == 3 && a.TS == 3 && abs(a.dth) == 1 && abs(a.dtw) == 1 && a.Cin % 8 == 0 && !a.resid;
}

static int64_t patches(const IgemmArgs &a)
{
    return (int64_t)a.NB * ((a.OH + P3_PH - 1) / P3_PH) * ((a.OW + P3_PW - 1) / P3_PW);
}

int64_t igemm_halo3x3_tiles(const IgemmArgs &a) { return patches(a) * ((a.Nout + P3_BN - 1) / P3_BN); }

namespace {
// How the output channels are cut into column tiles: n128 tiles of 128 channels, then n160 of 160,
// then at most one of <= 64.  Costs relative to a 128-wide tile (measured on the decoder layers): a
// 160-wide tile 1.25, the 64-wide kernel 0.7, a further launch 0.05.
struct ColumnPlan { int n128, n160, narrow; };
ColumnPlan plan_columns(int nout)
{
    ColumnPlan best{(nout + 127) / 128, 0, 0};
    double best_cost = 1e30;
    for (int n160 = 0; n160 <= (nout + 159) / 160; ++n160) {
        const int rest = nout - 160 * n160;
        int n128 = 0, narrow = 0;
        if (rest > 0) {
            n128 = rest / 128;
            const int r = rest - 128 * n128;
            if (r > 64) ++n128;
            else narrow = r;
        }
        const double cost = n128 + 1.25 * n160 + (narrow ? 0.7 : 0.0) + 0.05 * ((n128 > 0) + (n160 > 0) + (narrow > 0));
        if (cost < best_cost) { best_cost = cost; best = ColumnPlan{n128, n160, narrow}; }
    }
    return best;
}

template <int NB>
hipError_t launch_columns(const IgemmArgs &a, bool is_bf16, hipStream_t stream, int col_first, int ncols)
{
    constexpr int BN = 2 * NB * 16;
    const int64_t tiles = patches(a) * ((ncols + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    IgemmArgs w = a;
    w.Nout = ncols;
    w.D = a.D + col_first;
    if (a.bias) w.bias = a.bias + col_first;
    if (is_bf16) DLK_LAUNCH(kname("igemm_halo3x3_kernel", {NB}), (igemm_halo3x3_kernel<BF16, NB>), dim3((unsigned)tiles), dim3(512), 0, stream, w, col_first, a.Nout);
    else DLK_LAUNCH(kname("igemm_halo3x3_kernel", {NB}), (igemm_halo3x3_kernel<F16, NB>), dim3((unsigned)tiles), dim3(512), 0, stream, w, col_first, a.Nout);
    return dlk::launch_status();
}
}  // namespace

hipError_t launch_igemm_halo3x3(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    if (!igemm_halo3x3_applicable(a) || a.Nout <= 0) return hipErrorInvalidValue;
    const ColumnPlan cp = plan_columns(a.Nout);
    int col = 0;
    if (cp.n128 > 0) {
        const int n = min(a.Nout - col, cp.n128 * 128);
        const hipError_t e = launch_columns<4>(a, is_bf16, stream, col, n);
        if (e != hipSuccess) return e;
        col += n;
    }
    if (cp.n160 > 0) {
        const int n = min(a.Nout - col, cp.n160 * 160);
        const hipError_t e = launch_columns<5>(a, is_bf16, stream, col, n);
        if (e != hipSuccess) return e;
        col += n;
    }
    if (cp.narrow > 0) {
        const hipError_t e = launch_columns<2>(a, is_bf16, stream, col, cp.narrow);
        if (e != hipSuccess) return e;
        col += cp.narrow;
    }
    return col == a.Nout ? hipSuccess : hipErrorInvalidValue;
}

}  // namespace dlk
