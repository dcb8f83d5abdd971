// Implicit-GEMM convolution engine, direct-to-LDS variant (gfx950).
//
// Same GEMM view and tap addressing as the register-staged engine, but the
// activation and filter tiles travel global -> LDS without passing through
// registers: every wave issues `buffer_load_dwordx4 ... lds` instructions,
// each of which deposits 64 lanes x 16 bytes = 1 KB (16 tile rows of 32
// reduction elements) contiguously in LDS.  Out-of-range offsets (zero
// padding, ragged edges, steps past the end of the reduction) deposit zeros.
// A ring of four LDS buffers keeps three reduction steps in flight; one
// barrier per step.  Because the LDS image of a load is contiguous, bank
// conflicts are avoided by swizzling which 16-byte slice of a row each lane
// fetches instead of padding the row pitch.
//
// Two reduction orders:
//   tap-major      kk = (tap*Cin + c) runs linearly; a 32-deep step may
//                  straddle taps.  Any Cin % 8 == 0.
//   channel-major  for each 32-channel chunk all taps are visited in turn, so
//                  a workgroup re-reads the same few input rows tap after tap
//                  while they are cached, and everything that changes from
//                  step to step is wave-uniform: the per-lane work per load is
//                  one add and one select.  Whether a tap of a row falls into
//                  the padding is looked up in a per-row bit mask built once.
//                  A ragged last chunk is zero-filled.  Needs <= 64 taps.
#include "device_common.h"
#include "kernels.h"

namespace dlk {

// Row r of a tile is 64 bytes = 4 slices of 16 bytes.  Logical slice v of row
// r lives at physical slice v ^ ((r >> 2) & 3).  A 16-byte LDS read is served
// 16 lanes (256 bytes, 64 banks) per cycle; the 16 consecutive rows such a
// group reads at one logical slice then fall on 16 different 16-byte bank
// groups: 4*(r & 3) + (v ^ (r >> 2)).  (Measured: twice the read rate of the
// 2-way conflict of an 8-row rule, four times an unswizzled 64-byte pitch.)
__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }

typedef short bt_s16x4_t __attribute__((ext_vector_type(4)));

// BT: the filter operand is given reduction-major (see IgemmArgs::b_transposed); channel-major order only.
// Its tile is deposited as it lies in memory, [32 reduction channels][BN columns], 32-byte blocks of a
// row XOR-swizzled with the row index, and the MFMA fragments (8 consecutive reduction channels of one
// column per lane) come from ds_read_b64_tr_b16, as in the filter-gradient kernels.
// The body of the kernel: workgroup `tile` of the GEMM p (tiles are numbered column tile fastest),
// range `split` of a split reduction.
template <class T, int BM, int BN, int WM, int WN, bool CMAJOR, bool BT>
__device__ __forceinline__ void igemm_dma_tile(const IgemmArgs &p, const int tile, const int split)
{
    static_assert(!BT || CMAJOR, "a reduction-major filter needs the channel-major order");
    constexpr int NW = WM * WN;
    constexpr int STAGES = 4;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int AIW = BM / 16 / NW, BIW = BN / 16 / NW;   // load instructions per wave per step
    static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "every wave must issue the same number of loads");
    static_assert(TM >= 1 && TN >= 1, "wave tile too small");
    constexpr int IN_FLIGHT = (STAGES - 2) * (AIW + BIW);   // loads that may still be pending at the wait

    // Ring slots of both operands in one array; the epilogue re-uses it as staging space.
    __shared__ __align__(16) uint16_t lds[STAGES * (BM + BN) * BK];
    uint16_t *const sA0 = lds, *const sA1 = lds + BM * BK, *const sA2 = lds + 2 * BM * BK, *const sA3 = lds + 3 * BM * BK;
    uint16_t *const sB0 = lds + 4 * BM * BK, *const sB1 = sB0 + BN * BK, *const sB2 = sB0 + 2 * BN * BK, *const sB3 = sB0 + 3 * BN * BK;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int M = p.NB * p.OH * p.OW;
    const int NT = p.TR * p.TS;                       // taps
    const int Kred = NT * p.Cin;
    const int tiles_n = (p.Nout + BN - 1) / BN;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    const i32x4_t rsA = make_rsrc_words(p.A, (uint32_t)p.NB * p.IH * p.IW * p.Cin * 2u);
    const i32x4_t rsB = make_rsrc_words(p.B, BT ? (uint32_t)p.b_elems * 2u : (uint32_t)p.Nout * Kred * 2u);

    // ---- what this lane fetches: row (16*inst + lane/4), logical slice vec --
    const int lrow = lane >> 2;                          // row within a 16-row load
    const int vec = (lane & 3) ^ swz(lrow);              // same for every load of this lane
    int a_ih[AIW], a_iw[AIW];
    uint32_t a_off[AIW];                                 // byte offset of (row's tap (0,0) pixel, channel 8*vec)
    uint32_t a_mask_lo[AIW], a_mask_hi[AIW];             // channel-major: bit t = tap t of this row is inside the image
#pragma unroll
    for (int i = 0; i < AIW; ++i) {
        const int m = m0 + (wave + i * NW) * 16 + lrow;
        a_mask_lo[i] = a_mask_hi[i] = 0u;
        if (m < M) {
            const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
            const int oh = rem / p.OW, ow = rem - oh * p.OW;
            a_ih[i] = oh * p.sh + p.th0;
            a_iw[i] = ow * p.sw + p.tw0;
            a_off[i] = (uint32_t)(((n * p.IH + a_ih[i]) * p.IW + a_iw[i]) * p.Cin + vec * 8) * 2u;
            if constexpr (CMAJOR) {
                for (int t = 0; t < NT; ++t) {
                    const int jr = t / p.TS, js = t - jr * p.TS;
                    const int ih = a_ih[i] + jr * p.dth, iw = a_iw[i] + js * p.dtw;
                    const uint32_t in = ((unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW) ? 1u : 0u;
                    if (t < 32) a_mask_lo[i] |= in << t;
                    else a_mask_hi[i] |= in << (t - 32);
                }
            }
        } else {
            a_off[i] = 0;
            a_ih[i] = -(1 << 28);                        // fails every bounds test
            a_iw[i] = 0;
        }
    }
    uint32_t b_off[BIW];                                 // byte offset of (filter row, reduction index 8*vec)
    bool b_ok[BIW];
#pragma unroll
    for (int i = 0; i < BIW; ++i) {
        const int j = n0 + (wave + i * NW) * 16 + lrow;
        b_ok[i] = j < p.Nout;
        b_off[i] = ((uint32_t)j * (uint32_t)Kred + vec * 8) * 2u;
    }
    // reduction-major filter: a load covers RPI_B reduction rows of BN columns (LPR_B lanes of 16 bytes each);
    // load `inst` = wave + i*NW of a step holds rows inst*RPI_B .. +RPI_B-1, so row & 3 does not depend on i
    constexpr int LPR_B = BN / 8, RPI_B = 64 / LPR_B;
    constexpr int BT_SHIFT = BN >= 128 ? 1 : 0;          // rows of >= 8 blocks: spread 4 rows x 2 blocks over 8 bank ranges
    static_assert(!BT || (NW * RPI_B) % 4 == 0, "swizzle must not depend on the load index");
    const int bt_row = lane / LPR_B;                     // row within a load
    const int bt_row3 = (wave * RPI_B + bt_row) & 3;
    const int bt_pc = lane % LPR_B;                      // physical 16-byte chunk within the row
    const int bt_blk = BN >= 64 ? ((bt_pc >> 1) ^ (bt_row3 << BT_SHIFT)) : (bt_pc >> 1);
    const int bt_col = n0 + ((bt_blk << 1) | (bt_pc & 1)) * 8;
    const bool bt_ok = bt_col < p.Nout;

    // ---- reduction cursor ---------------------------------------------------
    // channel-major: (t, jr, js, c0) are wave-uniform; tap-major: (kk, c, js, jr) per lane
    // channels [c_first, c_end) of the reduction belong to this workgroup (all of them unless the reduction is split)
    int c_first = 0, c_end = p.Cin;
    if (CMAJOR && p.ksplits > 1) {
        c_first = split * p.split_chunks * BK;
        c_end = min(p.Cin, c_first + p.split_chunks * BK);
    }
    int t = 0, jr = 0, js = 0, c0 = c_first;
    int kk = vec * 8, c = 0;
    if constexpr (!CMAJOR) { c = kk % p.Cin; js = (kk / p.Cin) % p.TS; jr = (kk / p.Cin) / p.TS; }
    const int lane_c = vec * 8;

    // Issue the loads of the next reduction step into ring slot (sa, sb).
    auto issue = [&](uint16_t *sa, uint16_t *sb) {
        if constexpr (CMAJOR) {
            const uint32_t tap_a = (uint32_t)(((jr * p.dth) * p.IW + js * p.dtw) * p.Cin + c0) * 2u;   // uniform
            const uint32_t tap_b = (uint32_t)(t * p.Cin + c0) * 2u;                                    // uniform
            const bool cin = lane_c < c_end - c0;        // false only in a ragged last chunk / past the end
#pragma unroll
            for (int i = 0; i < AIW; ++i) {
                const uint32_t word = t < 32 ? a_mask_lo[i] : a_mask_hi[i];
                const bool ok = cin && ((word >> (t & 31)) & 1u);
                dma_load_16B(rsA, lds_addr(sa) + (wave + i * NW) * 16 * BK * 2, ok ? a_off[i] + tap_a : OOB_OFFSET);
            }
            if constexpr (BT) {
                const uint32_t tap_bt = (uint32_t)(p.b_base + jr * p.b_sr + js * p.b_ss + bt_col);     // per lane (column)
#pragma unroll
                for (int i = 0; i < BIW; ++i) {
                    const int k = c0 + (wave + i * NW) * RPI_B + bt_row;
                    dma_load_16B(rsB, lds_addr(sb) + (wave + i * NW) * 1024,
                                 (bt_ok && k < c_end) ? (tap_bt + (uint32_t)k * (uint32_t)p.b_ldk) * 2u : OOB_OFFSET);
                }
            } else {
#pragma unroll
                for (int i = 0; i < BIW; ++i)
                    dma_load_16B(rsB, lds_addr(sb) + (wave + i * NW) * 16 * BK * 2,
                                 (cin && b_ok[i]) ? b_off[i] + tap_b : OOB_OFFSET);
            }
            ++t;
            if (++js == p.TS) { js = 0; ++jr; }
            if (t == NT) { t = 0; jr = 0; js = 0; c0 += BK; }
        } else {
            const bool kin = kk < Kred;
            const int dh = jr * p.dth, dw = js * p.dtw;
            const uint32_t tap_a = (uint32_t)((dh * p.IW + dw) * p.Cin + (c - lane_c)) * 2u;
#pragma unroll
            for (int i = 0; i < AIW; ++i) {
                const int ih = a_ih[i] + dh, iw = a_iw[i] + dw;
                const bool ok = kin && (unsigned)ih < (unsigned)p.IH && (unsigned)iw < (unsigned)p.IW;
                dma_load_16B(rsA, lds_addr(sa) + (wave + i * NW) * 16 * BK * 2, ok ? a_off[i] + tap_a : OOB_OFFSET);
            }
#pragma unroll
            for (int i = 0; i < BIW; ++i)
                dma_load_16B(rsB, lds_addr(sb) + (wave + i * NW) * 16 * BK * 2,
                             (kin && b_ok[i]) ? b_off[i] + (uint32_t)(kk - lane_c) * 2u : OOB_OFFSET);
            kk += BK;
            c += BK;
            while (c >= p.Cin) {
                c -= p.Cin;
                if (++js == p.TS) { js = 0; ++jr; }
            }
        }
    };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment addressing: row (lane % 32) of a 32-row MFMA tile, slices 2*ks + lane/32
    const int frow = lane & 31;
    const int fsw = swz(frow);                           // tile bases are multiples of 32 rows
    int foff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) foff[ks] = frow * BK + (((ks * 2 + (lane >> 5)) ^ fsw) << 3);

    // MFMAs of one slot (two 16-deep slices); the fragments of both slices are
    // requested from LDS before the first MFMA is issued.
    // transpose-read addressing of a [32][BN] tile: lane = 16*g + q points at reduction row
    // 8*(g>>1) + 4*half + q/4 (+ 16*ks) and columns 16*(g&1) + 4*(q%4)..+3 of a 32-column MFMA tile
    const int tg = lane >> 4, tq = lane & 15;
    const int t_row = 8 * (tg >> 1) + (tq >> 2);
    const int t_sw = BN >= 64 ? ((t_row & 3) << BT_SHIFT) : 0;        // same for row + 4 and row + 16
    const int t_sub = 4 * (tq & 3), t_blk = tg & 1;
    auto load_frags = [&](u32x4_t (&a)[TM], u32x4_t (&b)[TN], const uint16_t *sa, const uint16_t *sb, int ks) {
        const uint16_t *wa = sa + wm * TM * 32 * BK + foff[ks];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const u32x4_t *>(wa + i * 32 * BK);
        if constexpr (BT) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int blk = ((wn * TN + j) * 2 + t_blk) ^ t_sw;
                const uint16_t *lo = sb + (16 * ks + t_row) * BN + blk * 16 + t_sub;
                const bt_s16x4_t l4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((bt_s16x4_t __attribute__((address_space(3))) *)lo);
                const bt_s16x4_t h4 =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((bt_s16x4_t __attribute__((address_space(3))) *)(lo + 4 * BN));
                const u32x2_t l2 = __builtin_bit_cast(u32x2_t, l4), h2 = __builtin_bit_cast(u32x2_t, h4);
                b[j][0] = l2[0]; b[j][1] = l2[1]; b[j][2] = h2[0]; b[j][3] = h2[1];
            }
        } else {
            const uint16_t *wb = sb + wn * TN * 32 * BK + foff[ks];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const u32x4_t *>(wb + j * 32 * BK);
        }
    };
    auto mma = [&](const uint16_t *sa, const uint16_t *sb) {
        u32x4_t fa[2][TM], fb[2][TN];
        load_frags(fa[0], fb[0], sa, sb, 0);
        load_frags(fa[1], fb[1], sa, sb, 1);
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = T::mfma(fb[s][j], fa[s][i], acc[i][j]);   // rows = output channels
    };

    // Wait until this wave's loads for the oldest pending step have landed,
    // then meet the other waves: after the barrier the step's tile is complete
    // in LDS and nobody still reads the slot that is refilled next.
    auto wait_and_sync = [&]() {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
    };

    // The step count is rounded up to a whole turn of the ring (the extra
    // steps load and multiply zeros) so that the unrolled loop has one exit.
    const int nk = CMAJOR ? ((c_end - c_first + BK - 1) / BK) * NT : (Kred + BK - 1) / BK;
    const int nturns = (nk + STAGES - 1) / STAGES;
    if (nk > 0) {
        issue(sA0, sB0);
        issue(sA1, sB1);
        issue(sA2, sB2);
        for (int turn = 0; turn < nturns; ++turn) {
            wait_and_sync(); issue(sA3, sB3); mma(sA0, sB0);
            wait_and_sync(); issue(sA0, sB0); mma(sA1, sB1);
            wait_and_sync(); issue(sA1, sB1); mma(sA2, sB2);
            wait_and_sync(); issue(sA2, sB2); mma(sA3, sB3);
        }
    }
    // every wave's loads (the trailing ones deposit zeros) and LDS reads are over before LDS is reused
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- epilogue ---------------------------------------------------------------
    // The filter rode in the first MFMA operand, so register v of lane l holds output
    // channel 8*(v/4) + 4*(l/32) + v%4 of tile row l%32: four consecutive channels per
    // register quartet.  Each wave rounds one 32-row slab of its tile at a time, parks it in a
    // private LDS area as [row][channel] (pitch: the wave's channels + 8 bytes, conflict-free
    // for the 8-byte writes) and writes it out 16 bytes per lane, whole rows of the wave's
    // channel range at a time.
    if (CMAJOR && p.ksplits > 1) {
        // split reduction: fp32 partial sums, four consecutive channels per store
        float *out = p.part + (size_t)split * M * p.Nout;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + (wm * TM + i) * 32 + (lane & 31);
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = n0 + (wn * TN + j) * 32 + 8 * g + 4 * (lane >> 5);
                    float *dst = out + (size_t)m * p.Nout + col;
                    if (col + 3 < p.Nout && (p.Nout & 3) == 0) {
                        floatx4_t v4;
                        v4[0] = acc[i][j][4 * g]; v4[1] = acc[i][j][4 * g + 1]; v4[2] = acc[i][j][4 * g + 2]; v4[3] = acc[i][j][4 * g + 3];
                        *reinterpret_cast<floatx4_t *>(dst) = v4;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < p.Nout) dst[e] = acc[i][j][4 * g + e];
                    }
                }
        }
        return;
    }
    constexpr int CH = TN * 32;                          // channels per wave
    constexpr int EP = CH + 4;                           // staging pitch in 16-bit elements
    constexpr int LPR = CH / 8;                          // lanes per row when writing out
    static_assert(NW * 32 * EP <= STAGES * (BM + BN) * BK, "staging area must fit the ring");
    uint16_t *stg = lds + wave * 32 * EP;
    const bool dense = (p.osh == 1 && p.osw == 1 && p.FH == p.OH && p.FW == p.OW);
    const bool vec_ok = (p.ldd % 8 == 0) && (p.Nout % 8 == 0) && ((reinterpret_cast<uintptr_t>(p.D) & 15) == 0);
    const bool tail = p.bias != nullptr || p.relu != 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // A residual input is added before the rounding.  Its 32-row slab is fetched the way the output is
        // written (16 bytes per lane, whole rows of the wave's channel range) into the staging area, and every
        // lane then picks up the four values that belong to its accumulators.
        if (p.resid) {
#pragma unroll
            for (int it = 0; it < LPR / 2; ++it) {
                const int row = it * (64 / LPR) + lane / LPR, c8 = (lane % LPR) * 8;
                const int m = m0 + (wm * TM + i) * 32 + row;
                const int col = n0 + wn * CH + c8;
                u32x2_t lo{0, 0}, hi{0, 0};
                if (m < M && col < p.Nout) {
                    size_t row_off;
                    if (dense) {
                        row_off = (size_t)m * p.ldd;
                    } else {
                        const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
                        const int oh = rem / p.OW, ow = rem - oh * p.OW;
                        row_off = ((size_t)(n * p.FH + oh * p.osh + p.ooh) * p.FW + ow * p.osw + p.oow) * p.ldd;
                    }
                    const uint16_t *src = p.resid + row_off + col;
                    if (vec_ok && (reinterpret_cast<uintptr_t>(p.resid) & 15) == 0) {
                        const u32x4_t v4 = *reinterpret_cast<const u32x4_t *>(src);
                        lo[0] = v4[0]; lo[1] = v4[1]; hi[0] = v4[2]; hi[1] = v4[3];
                    } else {
                        uint32_t w4[4] = {0, 0, 0, 0};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (col + e < p.Nout) w4[e >> 1] |= (uint32_t)src[e] << (16 * (e & 1));
                        lo[0] = w4[0]; lo[1] = w4[1]; hi[0] = w4[2]; hi[1] = w4[3];
                    }
                }
                *reinterpret_cast<u32x2_t *>(stg + row * EP + c8) = lo;
                *reinterpret_cast<u32x2_t *>(stg + row * EP + c8 + 4) = hi;
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = lane & 31, ch = j * 32 + 8 * g + 4 * (lane >> 5);
                floatx4_t c{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (p.resid) {
                    const u32x2_t r = *reinterpret_cast<const u32x2_t *>(stg + row * EP + ch);
                    c[0] += T::to_float((uint16_t)(r[0] & 0xffffu));
                    c[1] += T::to_float((uint16_t)(r[0] >> 16));
                    c[2] += T::to_float((uint16_t)(r[1] & 0xffffu));
                    c[3] += T::to_float((uint16_t)(r[1] >> 16));
                }
                if (tail) c = apply_tail4(c, p.bias, p.relu, n0 + wn * CH + ch, p.Nout);
                u32x2_t pk;
                pk[0] = (uint32_t)T::from_float(c[0]) | ((uint32_t)T::from_float(c[1]) << 16);
                pk[1] = (uint32_t)T::from_float(c[2]) | ((uint32_t)T::from_float(c[3]) << 16);
                *reinterpret_cast<u32x2_t *>(stg + row * EP + ch) = pk;
            }
#pragma unroll
        for (int it = 0; it < LPR / 2; ++it) {           // 32 rows x LPR lanes, 64 lanes at a time
            const int row = it * (64 / LPR) + lane / LPR, c8 = (lane % LPR) * 8;
            const u32x2_t lo = *reinterpret_cast<const u32x2_t *>(stg + row * EP + c8);
            const u32x2_t hi = *reinterpret_cast<const u32x2_t *>(stg + row * EP + c8 + 4);
            const int m = m0 + (wm * TM + i) * 32 + row;
            const int col = n0 + wn * CH + c8;
            if (m >= M || col >= p.Nout) continue;
            size_t row_off;
            if (dense) {
                row_off = (size_t)m * p.ldd;
            } else {
                const int n = m / (p.OH * p.OW), rem = m - n * (p.OH * p.OW);
                const int oh = rem / p.OW, ow = rem - oh * p.OW;
                row_off = ((size_t)(n * p.FH + oh * p.osh + p.ooh) * p.FW + ow * p.osw + p.oow) * p.ldd;
            }
            uint16_t *dst = p.D + row_off + col;
            if (vec_ok) {
                u32x4_t v4;
                v4[0] = lo[0]; v4[1] = lo[1]; v4[2] = hi[0]; v4[3] = hi[1];
                *reinterpret_cast<u32x4_t *>(dst) = v4;
            } else {
                const uint32_t w4[4] = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (col + e < p.Nout) dst[e] = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

template <class T, int BM, int BN, int WM, int WN, bool CMAJOR, bool BT = false>
__global__ __launch_bounds__(WM *WN * 64) void igemm_dma_kernel(const IgemmArgs p)
{
    // Split reduction into 2, 4 or 8 ranges: range s runs on the XCDs s, s + ranges, ... (workgroups are dealt to the
    // eight XCDs in turn, x fastest), so that an XCD's L2 holds one range of the channels of both operands
    // instead of all of them (ASPP 3x3 forward: 4.7 MB per XCD instead of 37 MB).
    if (gridDim.y > 1 && 8 % gridDim.y == 0) {
        const unsigned id = blockIdx.y * gridDim.x + blockIdx.x;
        igemm_dma_tile<T, BM, BN, WM, WN, CMAJOR, BT>(p, (int)(id / gridDim.y), (int)(id % gridDim.y));
        return;
    }
    igemm_dma_tile<T, BM, BN, WM, WN, CMAJOR, BT>(p, xcd_remap(blockIdx.x, gridDim.x), blockIdx.y);
}

// Several small GEMMs of one tile shape in one launch (the stride-parity classes of a strided
// data gradient on a small image, each of which alone is a ~10 us kernel): workgroup ids are
// dealt to the GEMMs in turn.  Channel-major order only.
template <class T, int BM, int BN, int WM, int WN, bool BT>
__global__ __launch_bounds__(WM *WN * 64) void igemm_dma_batch_kernel(const IgemmBatch b)
{
    const int id = xcd_remap(blockIdx.x, gridDim.x);
    const int which = id % b.n, tile = id / b.n;
    const IgemmArgs &p = b.a[which];
    const int64_t M = (int64_t)p.NB * p.OH * p.OW;
    const int64_t tiles = ((M + BM - 1) / BM) * ((p.Nout + BN - 1) / BN);
    if (tile >= tiles) return;                           // this GEMM has fewer tiles than the largest
    igemm_dma_tile<T, BM, BN, WM, WN, true, BT>(p, tile, 0);
}

template <class T, int BM, int BN, int WM, int WN>
static hipError_t launch_dma_cfg(const IgemmArgs &a, hipStream_t stream)
{
    const int64_t M = (int64_t)a.NB * a.OH * a.OW;
    const int64_t tiles = ((M + BM - 1) / BM) * ((a.Nout + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles, (unsigned)(a.c_outer && a.ksplits > 1 ? a.ksplits : 1)), block(WM * WN * 64);
    if (a.b_transposed) {
        if (!a.c_outer || a.Nout % 8 != 0) return hipErrorInvalidValue;
        DLK_LAUNCH(kname("igemm_dma_kernel.bt", {BM, BN}), (igemm_dma_kernel<T, BM, BN, WM, WN, true, true>), grid, block, 0, stream, a);
    } else if (a.c_outer)
        DLK_LAUNCH(kname("igemm_dma_kernel.cmajor", {BM, BN}), (igemm_dma_kernel<T, BM, BN, WM, WN, true>), grid, block, 0, stream, a);
    else
        DLK_LAUNCH(kname("igemm_dma_kernel.tapmajor", {BM, BN}), (igemm_dma_kernel<T, BM, BN, WM, WN, false>), grid, block, 0, stream, a);
    return dlk::launch_status();
}

template <class T>
static hipError_t dispatch_dma(const IgemmArgs &a, int cfg, hipStream_t stream)
{
    switch (cfg) {
        case 0: return launch_dma_cfg<T, 256, 256, 2, 4>(a, stream);   // 8 waves, wave tile 128x64
        case 2: return launch_dma_cfg<T, 128, 128, 2, 2>(a, stream);   // 4 waves, wave tile 64x64
        case 3: return launch_dma_cfg<T, 128, 64, 2, 2>(a, stream);    // 4 waves, wave tile 64x32
        case 4: return launch_dma_cfg<T, 64, 32, 2, 1>(a, stream);     // 2 waves, wave tile 32x32
        case 8: return launch_dma_cfg<T, 64, 64, 2, 1>(a, stream);     // 2 waves, wave tile 32x64
        default: return hipErrorInvalidValue;
    }
}

template <class T, int BM, int BN, int WM, int WN>
static hipError_t launch_dma_batch_cfg(const IgemmBatch &b, hipStream_t stream)
{
    int64_t tiles_max = 0;
    for (int i = 0; i < b.n; ++i) {
        const IgemmArgs &a = b.a[i];
        if (!a.c_outer || a.ksplits > 1 || a.b_transposed != b.a[0].b_transposed) return hipErrorInvalidValue;
        if (a.b_transposed && a.Nout % 8 != 0) return hipErrorInvalidValue;
        const int64_t M = (int64_t)a.NB * a.OH * a.OW;
        const int64_t tiles = ((M + BM - 1) / BM) * ((a.Nout + BN - 1) / BN);
        if (tiles > tiles_max) tiles_max = tiles;
    }
    if (tiles_max <= 0 || tiles_max * b.n > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(tiles_max * b.n)), block(WM * WN * 64);
    if (b.a[0].b_transposed) DLK_LAUNCH(kname("igemm_dma_batch_kernel.bt", {BM, BN}), (igemm_dma_batch_kernel<T, BM, BN, WM, WN, true>), grid, block, 0, stream, b);
    else DLK_LAUNCH(kname("igemm_dma_batch_kernel", {BM, BN}), (igemm_dma_batch_kernel<T, BM, BN, WM, WN, false>), grid, block, 0, stream, b);
    return dlk::launch_status();
}

template <class T>
static hipError_t dispatch_dma_batch(const IgemmBatch &b, int cfg, hipStream_t stream)
{
    switch (cfg) {
        case 0: return launch_dma_batch_cfg<T, 256, 256, 2, 4>(b, stream);
        case 2: return launch_dma_batch_cfg<T, 128, 128, 2, 2>(b, stream);
        case 3: return launch_dma_batch_cfg<T, 128, 64, 2, 2>(b, stream);
        case 4: return launch_dma_batch_cfg<T, 64, 32, 2, 1>(b, stream);
        case 8: return launch_dma_batch_cfg<T, 64, 64, 2, 1>(b, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_igemm_dma_batch(const IgemmBatch &b, bool is_bf16, int cfg, hipStream_t stream)
{
    if (b.n < 1 || b.n > IgemmBatch::MAX) return hipErrorInvalidValue;
    return is_bf16 ? dispatch_dma_batch<BF16>(b, cfg, stream) : dispatch_dma_batch<F16>(b, cfg, stream);
}

hipError_t launch_igemm_dma(const IgemmArgs &a, bool is_bf16, int cfg, hipStream_t stream)
{
    return is_bf16 ? dispatch_dma<BF16>(a, cfg, stream) : dispatch_dma<F16>(a, cfg, stream);
}

}  // namespace dlk
