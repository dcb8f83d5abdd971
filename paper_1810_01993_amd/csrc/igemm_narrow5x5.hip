// Halo-tile implicit-GEMM kernels for dense 5x5 filters with unit stride and
// dilation where one side of the layer has at most 32 channels (gfx950): the
// dense-block layers of a Tiramisu-style network (growth rate 32).  First the
// forward pass (at most 32 OUTPUT channels), where a 256- or 128-wide column
// tile would be mostly padding and the plain engine re-fetches the activation
// tile from L2 for each of the 25 taps; further down its mirror image, the
// data gradient (at most 32 channels on the reduction side).
//
// A workgroup (4 waves) owns a 16-row x 32-column patch of output pixels and
// all output channels; wave w owns patch rows 4w .. 4w+3.  Per 32-channel
// chunk of the input the patch with its halo (20 x 36 pixels, 45 KB) is
// deposited in LDS once and serves all 25 taps.  Taps are visited column shift
// by column shift: for one column shift a wave reads the eight halo rows under
// its four patch rows once (16 fragments) and the five filter taps of that
// column (10 fragments) and issues 80 MFMAs, each halo row serving up to five
// row shifts from registers: 0.33 LDS fragment reads per MFMA.
//
// The five filter taps of a column shift (10 KB) travel through a ring of three
// LDS slots, two column shifts ahead.  The halo image is single-buffered (two
// workgroups of 79 KB share a compute unit, and a second image would not fit):
// the next chunk's image is requested as soon as every wave has read its
// fragments of the chunk's last column shift, so the 80 MFMAs of that shift and
// the other workgroup's work cover most of its latency.  Every step issues the
// same number of loads per wave (stand-ins go to a spare area), so one constant
// wait count serves: when a step starts, everything but the newest filter slot
// has landed.
#include <algorithm>
#include <cstdlib>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

namespace {
constexpr int N5_PH = 16, N5_PW = 32, N5_T = 5, N5_BN = 32;
constexpr int N5_HH = N5_PH + N5_T - 1, N5_HW = N5_PW + N5_T - 1;       // 20 x 36
__device__ __forceinline__ int n5_swz(int row) { return (row >> 1) & 3; }   // 16-row operands: conflict-free at any alignment
}  // namespace

template <class T>
__global__ __launch_bounds__(256, 2) void igemm_narrow5x5_kernel(const IgemmArgs p)
{
    constexpr int NW = 4, TM = 4, NT = N5_T * N5_T, KB = N5_BN / 16;
    constexpr int HW = N5_HW, HH = N5_HH;
    constexpr int HPIECES = (HH * HW + 15) / 16;         // 45 pieces of 16 halo pixels
    constexpr int AW = (HPIECES + NW - 1) / NW;          // halo loads per wave per chunk (stand-ins included)
    constexpr int FPIECES = N5_T * KB;                   // 10 pieces of 16 filter rows per column shift
    constexpr int FW = (FPIECES + NW - 1) / NW;          // filter loads per wave per step (stand-ins included)
    constexpr int S = 3;                                 // filter ring slots
    constexpr int H_ELEMS = HPIECES * 16 * BK, F_ELEMS = FPIECES * 16 * BK, SPARE_ELEMS = NW * 16 * BK;
    __shared__ __align__(16) uint16_t lds[H_ELEMS + S * F_ELEMS + SPARE_ELEMS];
    uint16_t *const sH = lds, *const sF = lds + H_ELEMS, *const sSpare = sF + S * F_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nchunks = (p.Cin + BK - 1) / BK;
    // Split reduction (maps with few patches): gridDim.y workgroups per patch, workgroup z takes the chunks
    // [z * split_chunks, ...) and writes fp32 partial sums part[z][pixel][column] for the ordered reduce.
    const int chunk_begin = p.ksplits > 1 ? (int)blockIdx.y * p.split_chunks : 0;
    const int chunk_end = p.ksplits > 1 ? min(nchunks, chunk_begin + p.split_chunks) : nchunks;

    const int tiles_x = (p.OW + N5_PW - 1) / N5_PW, tiles_y = (p.OH + N5_PH - 1) / N5_PH;
    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tx = tile % tiles_x; tile /= tiles_x;
    const int ty = tile % tiles_y;
    const int img = tile / tiles_y;
    const int y0 = ty * N5_PH, x0 = tx * N5_PW;

    const i32x4_t rsA = make_rsrc_words(p.A, (uint32_t)p.NB * p.IH * p.IW * p.Cin * 2u);
    const i32x4_t rsB = make_rsrc_words(p.B, (uint32_t)nchunks * NT * p.Nout * BK * 2u);

    // ---- what this lane fetches ---------------------------------------------
    const int lrow = lane >> 2;
    const int lane_c = ((lane & 3) ^ n5_swz(lrow)) * 8;
    uint32_t h_off[AW];                                  // byte offset of (halo pixel, channel lane_c), or out of range
#pragma unroll
    for (int a = 0; a < AW; ++a) {
        const int pc = wave + a * NW;
        const int hp = pc * 16 + lrow;
        const int hy = hp / HW, hx = hp - hy * HW;
        const int iy = y0 + p.th0 + hy, ix = x0 + p.tw0 + hx;
        const bool ok = pc < HPIECES && hy < HH && (unsigned)iy < (unsigned)p.IH && (unsigned)ix < (unsigned)p.IW;
        h_off[a] = ok ? (uint32_t)(((img * p.IH + iy) * p.IW + ix) * p.Cin + lane_c) * 2u : OOB_OFFSET;
    }
    // filter piece wave + f*NW of a column shift: tap row (piece / KB), output channels 16*(piece % KB) ..
    uint32_t b_off[FW];                                  // offset within the (chunk, column shift), or out of range
#pragma unroll
    for (int f = 0; f < FW; ++f) {
        const int pc = wave + f * NW;
        const int tr = pc / KB, j = 16 * (pc % KB) + lrow;
        b_off[f] = (pc < FPIECES && j < p.Nout) ? (uint32_t)((tr * N5_T * p.Nout + j) * BK + lane_c) * 2u : OOB_OFFSET;
    }
    auto issue_halo = [&](int chunk) {                   // the whole image of a chunk (zeros past the last channel / chunk)
        const int c0 = chunk * BK;
#pragma unroll
        for (int a = 0; a < AW; ++a) {
            const int pc = wave + a * NW;
            const uint32_t dst = pc < HPIECES ? lds_addr(sH) + pc * 16 * BK * 2 : lds_addr(sSpare) + wave * 16 * BK * 2;
            dma_load_16B(rsA, dst, (h_off[a] != OOB_OFFSET && chunk < chunk_end && lane_c < p.Cin - c0) ? h_off[a] + (uint32_t)c0 * 2u : OOB_OFFSET);
        }
    };
    auto issue_filter = [&](int g) {                     // column shift g % 5 of chunk g / 5, into slot g % 3
        const int chunk = g / N5_T, cs = g - chunk * N5_T, slot = g % S;
        const uint32_t base = (uint32_t)((chunk * NT + cs) * p.Nout) * (BK * 2u);   // past the last chunk: out of range
#pragma unroll
        for (int f = 0; f < FW; ++f) {
            const int pc = wave + f * NW;
            const uint32_t dst = pc < FPIECES ? lds_addr(sF + slot * F_ELEMS) + pc * 16 * BK * 2 : lds_addr(sSpare) + wave * 16 * BK * 2;
            dma_load_16B(rsB, dst, (b_off[f] != OOB_OFFSET && chunk < chunk_end) ? b_off[f] + base : OOB_OFFSET);
        }
    };

    // acc[i][kb][b]: patch row i of the wave, 16-channel block kb, pixel half b of the row
    floatx4_t acc[TM][KB][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[i][kb][b] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    // an operand tile is 16 rows (channels or pixels) x 32 reduction elements: lane l reads the
    // 16-byte slice l/16 of row l%16
    const int frow = lane & 15, fsl = lane >> 4;
    const int foff = frow * BK + ((fsl ^ n5_swz(frow)) << 3);
    const int hbase = (wave * TM) * HW + frow;

    issue_halo(chunk_begin);
    issue_filter(chunk_begin * N5_T);
    issue_filter(chunk_begin * N5_T + 1);
    const int nsteps = chunk_end * N5_T;
    for (int g = chunk_begin * N5_T, cs = 0; g < nsteps; ++g) {
        // everything but the newest filter slot has landed; every wave is past the previous step's reads
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(FW) : "memory");
        __builtin_amdgcn_sched_barrier(0);
        if (cs != N5_T - 1) issue_filter(g + 2);         // into the slot the previous step read
        u32x4_t fa[TM + N5_T - 1][2], fb[N5_T][KB];
#pragma unroll
        for (int r = 0; r < TM + N5_T - 1; ++r)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int h = hbase + r * HW + cs + 16 * b;
                fa[r][b] = *reinterpret_cast<const u32x4_t *>(sH + h * BK + ((fsl ^ n5_swz(h)) << 3));
            }
        const uint16_t *wb = sF + (g % S) * F_ELEMS + foff;
#pragma unroll
        for (int tr = 0; tr < N5_T; ++tr)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) fb[tr][kb] = *reinterpret_cast<const u32x4_t *>(wb + (tr * KB + kb) * 16 * BK);
        if (cs == N5_T - 1) {
            // last column shift of the chunk: once every wave holds its fragments the image can be replaced
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            issue_halo(g / N5_T + 1);
            issue_filter(g + 2);
        }
#pragma unroll
        for (int tr = 0; tr < N5_T; ++tr)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int b = 0; b < 2; ++b) T::mfma16_acc(acc[i][kb][b], fb[tr][kb], fa[i + tr][b]);   // rows = channels
        cs = cs == N5_T - 1 ? 0 : cs + 1;
    }
    // every wave's loads (the trailing ones deposit zeros) and LDS reads are over before LDS is reused
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    mfma_acc_settle();

    // ---- epilogue ---------------------------------------------------------------
    // The filter rode in the first MFMA operand, so register v of lane l of a 16x16 block holds
    // channel 4*(l/16) + v of pixel l%16.  Each wave rounds its 4 rows x 32 pixels x 32 channels to
    // 16 bits, parks them in a private LDS area as [pixel][channel] (pitch 80 bytes: an odd number
    // of 16-byte units) and writes them out 16 bytes per lane; with 32 output channels a patch row
    // is one contiguous 2 KB run.
    if (p.ksplits > 1) {
        // fp32 partial sums, four consecutive channels per store; bias, activation and rounding happen in the reduce
        const int64_t M = (int64_t)p.NB * p.OH * p.OW;
        float *const out = p.part + (size_t)blockIdx.y * M * p.Nout;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int y = y0 + wave * TM + i, x = x0 + b * 16 + (lane & 15);
                if (y >= p.OH || x >= p.OW) continue;
                float *row = out + ((size_t)(img * p.OH + y) * p.OW + x) * p.Nout;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const int col = kb * 16 + 4 * (lane >> 4);
                    if (col < p.Nout) *reinterpret_cast<floatx4_t *>(row + col) = acc[i][kb][b];     // Nout % 8 == 0
                }
            }
        return;
    }
    constexpr int EP = N5_BN + 8;
    static_assert((EP / 8) % 2 == 1 && NW * TM * N5_PW * EP <= H_ELEMS, "staging area");
    uint16_t *const stg = lds + wave * (TM * N5_PW) * EP;
    const bool tail = p.bias != nullptr || p.relu != 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                floatx4_t c = acc[i][kb][b];
                if (tail) c = apply_tail4(c, p.bias, p.relu, kb * 16 + 4 * (lane >> 4), p.Nout);
                u32x2_t pk;
                pk[0] = (uint32_t)T::from_float(c[0]) | ((uint32_t)T::from_float(c[1]) << 16);
                pk[1] = (uint32_t)T::from_float(c[2]) | ((uint32_t)T::from_float(c[3]) << 16);
                const int px = i * N5_PW + b * 16 + (lane & 15), ch = kb * 16 + 4 * (lane >> 4);
                *reinterpret_cast<u32x2_t *>(stg + px * EP + ch) = pk;
            }
    constexpr int LPR = N5_BN / 8;                       // lanes per pixel when writing out
#pragma unroll
    for (int it = 0; it < TM * N5_PW * LPR / 64; ++it) {
        const int item = it * 64 + lane;
        const int px = item / LPR, c8 = (item % LPR) * 8;
        const u32x4_t v4 = *reinterpret_cast<const u32x4_t *>(stg + px * EP + c8);
        const int y = y0 + wave * TM + px / N5_PW, x = x0 + px % N5_PW;
        if (y >= p.OH || x >= p.OW || c8 >= p.Nout) continue;
        *reinterpret_cast<u32x4_t *>(p.D + ((size_t)(img * p.OH + y) * p.OW + x) * p.ldd + c8) = v4;
    }
}

// ---- the mirror case: at most 32 INPUT channels, many output columns ------------------------
// The data gradient of such a layer (dx of C channels from dy of 32) has a single 32-channel
// chunk of reduction, so a tile of the kernels above would be 25 steps long and mostly set-up.
// Here a workgroup (4 waves, wave w = patch rows 4w .. 4w+3) deposits the halo image of its
// 16 x 32 patch once and then produces ALL output columns, 64 at a time: per column tile 25
// steps (one tap each, 4 KB of filter through a ring of six LDS slots, four steps in flight),
// the 16 halo-row fragments re-read once per column shift and kept for its five row shifts,
// 32 MFMAs per step and wave.  Blocks of 16 columns beyond the last are skipped, not padded.
// The accumulators go straight to memory (a lane holds four consecutive channels of a pixel:
// 8-byte stores; the four blocks of a pixel complete a 128-byte line in L2).
// Taps may be mirrored (data gradient) or not.
template <class T>
__global__ __launch_bounds__(256, 2) void igemm_wide5x5_kernel(const IgemmArgs p)
{
    constexpr int NW = 4, TM = 4, KB = 4, BN = KB * 16;
    constexpr int HW = N5_HW, HH = N5_HH;
    constexpr int HPIECES = (HH * HW + 15) / 16;         // 45 pieces of 16 halo pixels
    constexpr int AW = (HPIECES + NW - 1) / NW;          // halo loads per wave (stand-ins included)
    constexpr int S = 6, IN_FLIGHT = S - 2;              // filter ring; one load per wave per step
    constexpr int H_ELEMS = HPIECES * 16 * BK, F_ELEMS = BN * BK, SPARE_ELEMS = NW * 16 * BK;
    __shared__ __align__(16) uint16_t lds[H_ELEMS + S * F_ELEMS + SPARE_ELEMS];
    uint16_t *const sH = lds, *const sF = lds + H_ELEMS, *const sSpare = sF + S * F_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool flip_r = p.dth < 0, flip_s = p.dtw < 0;   // which tap a given shift belongs to
    const int oy_min = flip_r ? p.th0 - (N5_T - 1) : p.th0, ox_min = flip_s ? p.tw0 - (N5_T - 1) : p.tw0;

    const int tiles_x = (p.OW + N5_PW - 1) / N5_PW, tiles_y = (p.OH + N5_PH - 1) / N5_PH;
    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tx = tile % tiles_x; tile /= tiles_x;
    const int ty = tile % tiles_y;
    const int img = tile / tiles_y;
    const int y0 = ty * N5_PH, x0 = tx * N5_PW;
    const int ntiles_n = (p.Nout + 63) / 64;

    const i32x4_t rsA = make_rsrc_words(p.A, (uint32_t)p.NB * p.IH * p.IW * p.Cin * 2u);
    const i32x4_t rsB = make_rsrc_words(p.B, (uint32_t)(N5_T * N5_T) * p.Nout * BK * 2u);

    const int lrow = lane >> 2;
    const int lane_c = ((lane & 3) ^ n5_swz(lrow)) * 8;
    // ---- the halo image, once -------------------------------------------------------
#pragma unroll
    for (int a = 0; a < AW; ++a) {
        const int pc = wave + a * NW;
        const int hp = pc * 16 + lrow;
        const int hy = hp / HW, hx = hp - hy * HW;
        const int iy = y0 + oy_min + hy, ix = x0 + ox_min + hx;
        const bool ok = pc < HPIECES && hy < HH && (unsigned)iy < (unsigned)p.IH && (unsigned)ix < (unsigned)p.IW && lane_c < p.Cin;
        const uint32_t dst = pc < HPIECES ? lds_addr(sH) + pc * 16 * BK * 2 : lds_addr(sSpare) + wave * 16 * BK * 2;
        dma_load_16B(rsA, dst, ok ? (uint32_t)(((img * p.IH + iy) * p.IW + ix) * p.Cin + lane_c) * 2u : OOB_OFFSET);
    }
    // ---- the filter stream: step g = (column tile, column shift, row shift) -----------------
    // this wave's piece of a tap tile: rows (output columns) 16*wave + lrow of the column tile
    // (with few patches the column tiles are dealt over gridDim.y workgroups per patch: this one takes tiles
    // blockIdx.y, blockIdx.y + gridDim.y, ...)
    int ld_ct = blockIdx.y, ld_cs = 0, ld_tr = 0;
    auto issue_filter = [&](int slot) {
        const int jr = flip_r ? N5_T - 1 - ld_tr : ld_tr, js = flip_s ? N5_T - 1 - ld_cs : ld_cs;
        const int j = ld_ct * BN + 16 * wave + lrow;
        const bool ok = ld_ct < ntiles_n && j < p.Nout;
        dma_load_16B(rsB, lds_addr(sF + slot * F_ELEMS) + wave * 16 * BK * 2,
                     ok ? (uint32_t)(((jr * N5_T + js) * p.Nout + j) * BK + lane_c) * 2u : OOB_OFFSET);
        if (++ld_tr == N5_T) {
            ld_tr = 0;
            if (++ld_cs == N5_T) { ld_cs = 0; ld_ct += gridDim.y; }
        }
    };

    floatx4_t acc[TM][KB][2];
    auto clear_acc = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[i][kb][b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    };
    clear_acc();

    const int frow = lane & 15, fsl = lane >> 4;
    const int foff = frow * BK + ((fsl ^ n5_swz(frow)) << 3);
    const int hbase = (wave * TM) * HW + frow;
    const bool tail = p.bias != nullptr || p.relu != 0;

#pragma unroll
    for (int k = 0; k < S - 1; ++k) issue_filter(k);
    int slot = 0;
    for (int ct = blockIdx.y; ct < ntiles_n; ct += gridDim.y) {
        const int nblk = min(KB, (p.Nout - ct * BN + 15) / 16);     // 16-column blocks of this tile that exist
#pragma unroll
        for (int cs = 0; cs < N5_T; ++cs) {
            u32x4_t fa[TM + N5_T - 1][2];
#pragma unroll
            for (int tr = 0; tr < N5_T; ++tr) {
                // this wave's load for the step has landed (four later ones may be in flight); after the
                // barrier everybody's has, and every wave is past its reads of the previous step's slot
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(IN_FLIGHT) : "memory");
                __builtin_amdgcn_sched_barrier(0);
                issue_filter(slot == 0 ? S - 1 : slot - 1);
                if (tr == 0) {
                    // (from opaque copies, so that the 40 fragment addresses of a column tile are computed
                    // here, 8 at a time, and not kept in registers across the whole loop)
                    int hb = hbase, sl = fsl;
                    asm volatile("" : "+v"(hb), "+v"(sl));
#pragma unroll
                    for (int r = 0; r < TM + N5_T - 1; ++r)
#pragma unroll
                        for (int b = 0; b < 2; ++b) {
                            const int h = hb + r * HW + cs + 16 * b;
                            fa[r][b] = *reinterpret_cast<const u32x4_t *>(sH + h * BK + ((sl ^ n5_swz(h)) << 3));
                        }
                }
                u32x4_t fb[KB];
                const uint16_t *wb = sF + slot * F_ELEMS + foff;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) fb[kb] = *reinterpret_cast<const u32x4_t *>(wb + kb * 16 * BK);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
                    if (kb < nblk) {
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int b = 0; b < 2; ++b) T::mfma16_acc(acc[i][kb][b], fb[kb], fa[i + tr][b]);   // rows = channels
                    }
                slot = slot + 1 == S ? 0 : slot + 1;
            }
        }
        // ---- the column tile is complete: register v of lane l of a block holds channel 4*(l/16) + v of pixel l%16
        mfma_acc_settle();
        // (addressing from a copy of the lane number the optimiser cannot see through: computed before the
        // loop, the eight pixel addresses would occupy registers the steps need)
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int col = ct * BN + kb * 16 + 4 * (ln >> 4);
            if (kb >= nblk || col >= p.Nout) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    floatx4_t c = acc[i][kb][b];
                    if (tail) c = apply_tail4(c, p.bias, p.relu, col, p.Nout);
                    const int y = y0 + wave * TM + i, x = x0 + b * 16 + (ln & 15);
                    if (y >= p.OH || x >= p.OW) continue;
                    u32x2_t pk;
                    pk[0] = (uint32_t)T::from_float(c[0]) | ((uint32_t)T::from_float(c[1]) << 16);
                    pk[1] = (uint32_t)T::from_float(c[2]) | ((uint32_t)T::from_float(c[3]) << 16);
                    *reinterpret_cast<u32x2_t *>(p.D + ((size_t)(img * p.OH + y) * p.OW + x) * p.ldd + col) = pk;
                }
        }
        clear_acc();
    }
    // the trailing filter loads (zeros) land before the workgroup gives its LDS back
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

static int64_t narrow_tiles(const IgemmArgs &a)
{
    return (int64_t)a.NB * ((a.OH + N5_PH - 1) / N5_PH) * ((a.OW + N5_PW - 1) / N5_PW);
}

// Maps with fewer than 128 patches: how many ranges the 32-channel chunks are cut into (1: no split) so that
// the launch has about two workgroups per CU; *chunks_per_split: chunks per range.
static int narrow_ksplits(const IgemmArgs &a, int *chunks_per_split)
{
    const int nchunks = (a.Cin + BK - 1) / BK;
    const int64_t tiles = narrow_tiles(a);
    int ks = 1;
    if (tiles < 128 && a.ldd == a.Nout) ks = (int)std::min<int64_t>(nchunks, (512 + tiles - 1) / tiles);
    const int cps = (nchunks + ks - 1) / ks;
    ks = (nchunks + cps - 1) / cps;                      // no empty range
    if (chunks_per_split) *chunks_per_split = cps;
    return ks;
}

size_t igemm_narrow5x5_split_bytes(const IgemmArgs &a)
{
    const int ks = narrow_ksplits(a, nullptr);
    return ks > 1 ? (size_t)ks * a.NB * a.OH * a.OW * a.Nout * sizeof(float) : 0;
}

// Forward-oriented taps only (a data gradient of such a layer has 32 INPUT channels and many
// output columns: not this kernel's shape).
bool igemm_narrow5x5_applicable(const IgemmArgs &a)
{
    static const int mode = tuning_knob("DLCONV_NARROW", 1); // tuning override: 0 = never
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW;
    return mode && dense && a.TR == N5_T && a.TS == N5_T && a.dth == 1 && a.dtw == 1 && a.Cin % 8 == 0 &&
           a.Nout % 8 == 0 && a.Nout >= 8 && a.Nout <= N5_BN && a.ldd % 8 == 0 && !a.resid &&
           narrow_tiles(a) * narrow_ksplits(a, nullptr) >= 128;
}

// At most 32 input channels (one chunk), any number (a multiple of 4) of output columns, taps forward or mirrored.
bool igemm_wide5x5_applicable(const IgemmArgs &a)
{
    static const int mode = tuning_knob("DLCONV_WIDE5X5", 1); // tuning override: 0 = never
    const bool dense = a.sh == 1 && a.sw == 1 && a.osh == 1 && a.osw == 1 && a.FH == a.OH && a.FW == a.OW;
    return mode && dense && a.TR == N5_T && a.TS == N5_T && abs(a.dth) == 1 && abs(a.dtw) == 1 && a.Cin % 8 == 0 &&
           a.Cin <= BK && a.Nout % 4 == 0 && a.Nout > N5_BN && a.ldd % 4 == 0 && !a.resid &&
           narrow_tiles(a) * ((a.Nout + 63) / 64) >= 128;
}

hipError_t launch_igemm_wide5x5(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t tiles = narrow_tiles(a);
    if (!igemm_wide5x5_applicable(a) || tiles > 0x7fffffff || (reinterpret_cast<uintptr_t>(a.D) & 7) != 0) return hipErrorInvalidValue;
    // enough workgroups for the chip (two per CU): with few patches the column tiles of a patch are dealt
    // over several workgroups, each of which deposits the halo image for itself
    const int ntiles_n = (a.Nout + 63) / 64;
    const int per_patch = (int)std::min<int64_t>(ntiles_n, std::max<int64_t>(1, 512 / tiles));
    const dim3 grid((unsigned)tiles, (unsigned)per_patch);
    if (is_bf16) DLK_LAUNCH("igemm_wide5x5_kernel", igemm_wide5x5_kernel<BF16>, grid, dim3(256), 0, stream, a);
    else DLK_LAUNCH("igemm_wide5x5_kernel", igemm_wide5x5_kernel<F16>, grid, dim3(256), 0, stream, a);
    return dlk::launch_status();
}

hipError_t launch_igemm_narrow5x5(const IgemmArgs &a, bool is_bf16, hipStream_t stream)
{
    const int64_t tiles = narrow_tiles(a);
    if (!igemm_narrow5x5_applicable(a) || tiles > 0x7fffffff || (reinterpret_cast<uintptr_t>(a.D) & 15) != 0) return hipErrorInvalidValue;
    IgemmArgs b = a;
    int cps = 0;
    const int ks = narrow_ksplits(a, &cps);
    b.ksplits = ks;
    b.split_chunks = cps;
    if (ks > 1 && !a.part) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles, (unsigned)ks);
    if (is_bf16) DLK_LAUNCH("igemm_narrow5x5_kernel", igemm_narrow5x5_kernel<BF16>, grid, dim3(256), 0, stream, b);
    else DLK_LAUNCH("igemm_narrow5x5_kernel", igemm_narrow5x5_kernel<F16>, grid, dim3(256), 0, stream, b);
    hipError_t e = dlk::launch_status();
    if (e != hipSuccess || ks == 1) return e;
    return launch_splitk_reduce_tail(a.part, ks, (int64_t)a.NB * a.OH * a.OW * a.Nout, a.D, is_bf16 ? 1 : 0, a.bias, a.relu,
                                     a.Nout, nullptr, stream);
}

}  // namespace dlk
