// Data gradient of a 7x7, stride-2, padding-3 convolution with few input
// channels (gfx950): the network's stem, dx[N,H,W,16] from dy[N,H/2,W/2,64].
//
// As four stride-parity GEMMs with 16 output columns this layer is bound by
// the L2 -> LDS traffic of the activation operand: every tap re-fetches its
// dy tile and each fetched element meets only 16 columns.  Here a workgroup
// owns a 16 x 16 patch of dy pixels and produces the 32 x 32 output pixels
// (all four parity classes) they map to.  It deposits, once,
//   - the patch with its halo (19 x 19 dy pixels: output pixel (2p+a, 2q+b)
//     takes dy rows p-1 .. p+2) for every 32-channel chunk of K (at most two),
//   - the whole filter, re-laid-out as [chunk][tap][16 c][32 k],
// in LDS (47 KB + 98 KB), waits, and then runs without any further
// synchronisation: a wave owns two dy rows and all four classes of them
// (8 accumulators of 16 pixels x 16 channels), keeps the 5 rows x 4 column
// shifts of dy fragments it needs for a chunk in registers (each serves ~5 of
// the 98 (class, tap, row) products) and reads one filter fragment per tap.
// The filter rides in the first MFMA operand, so a lane ends up with four
// consecutive channels of one pixel; the 32 x 32 x 16 tile is assembled in LDS
// and written out as whole 1 KB rows.
#include <cstdlib>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

namespace {
constexpr int DS_R = 7, DS_PAD = 3;
constexpr int DS_TP = 16;                                // dy patch edge
constexpr int DS_HW = DS_TP + 3;                         // halo edge: rows p0 - 1 .. p0 + 17
constexpr int DS_PIECES = (DS_HW * DS_HW + 15) / 16;     // 16-pixel pieces of the halo image
constexpr int DS_MAXCH = 2;                              // 32-channel chunks of K held at once
__device__ __forceinline__ int ds_swz(int row) { return (row >> 1) & 3; }   // 16-row operands: conflict-free at any alignment
}  // namespace

template <class T>
__global__ __launch_bounds__(512) void dgrad_stem_kernel(const DgradStemArgs p)
{
    constexpr int NW = 8, NT = DS_R * DS_R;
    constexpr int H_ELEMS = DS_PIECES * 16 * BK;         // one chunk's halo image
    constexpr int F_ELEMS = NT * 16 * BK;                // one chunk's filter
    __shared__ __align__(16) uint16_t lds[DS_MAXCH * (H_ELEMS + F_ELEMS)];
    uint16_t *const sD = lds, *const sF = lds + DS_MAXCH * H_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nchunks = (p.K + BK - 1) / BK;             // <= DS_MAXCH (checked by the host)
    const int PH = (p.H + 1) / 2, PW = (p.W + 1) / 2;    // class-pixel grid that covers the output
    const int tiles_x = (PW + DS_TP - 1) / DS_TP, tiles_y = (PH + DS_TP - 1) / DS_TP;
    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tx = tile % tiles_x; tile /= tiles_x;
    const int ty = tile % tiles_y;
    const int img = tile / tiles_y;
    const int p0 = ty * DS_TP, q0 = tx * DS_TP;

    // ---- deposit the halo images and the filter ---------------------------------
    const i32x4_t rsD = make_rsrc_words(p.dy, (uint32_t)p.N * p.P * p.Q * p.K * 2u);
    const i32x4_t rsF = make_rsrc_words(p.wblk, (uint32_t)nchunks * NT * p.C * BK * 2u);
    const int lrow = lane >> 2;
    for (int piece = wave; piece < nchunks * DS_PIECES; piece += NW) {
        const int ch = piece / DS_PIECES, pc = piece - ch * DS_PIECES;
        const int hp = pc * 16 + lrow;                   // halo pixel
        const int hy = hp / DS_HW, hx = hp - hy * DS_HW;
        const int py = p0 - 1 + hy, px = q0 - 1 + hx;
        const int k = ch * BK + (((lane & 3) ^ ds_swz(hp)) << 3);
        const bool ok = hy < DS_HW && (unsigned)py < (unsigned)p.P && (unsigned)px < (unsigned)p.Q && k < p.K;
        dma_load_16B(rsD, lds_addr(sD + ch * H_ELEMS) + pc * 1024,
                     ok ? (uint32_t)(((img * p.P + py) * p.Q + px) * p.K + k) * 2u : OOB_OFFSET);
    }
    for (int piece = wave; piece < nchunks * NT; piece += NW) {
        // rows = output channels c (16 per tile; those at or beyond C read as zeros)
        const int kk = ((lane & 3) ^ ds_swz(lrow)) << 3;
        dma_load_16B(rsF, lds_addr(sF) + piece * 1024,
                     lrow < p.C ? (uint32_t)((piece * p.C + lrow) * BK + kk) * 2u : OOB_OFFSET);
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- products ----------------------------------------------------------------
    // acc[a][b][i]: parity class (a, b), dy row 2*wave + i of the patch
    floatx4_t acc[2][2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 2; ++i) acc[a][b][i] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    const int frow = lane & 15, fsl = lane >> 4;
    const int foff = frow * BK + ((fsl ^ ds_swz(frow)) << 3);          // within a filter tile
    for (int ch = 0; ch < nchunks; ++ch) {
        // dy fragments: halo rows 2*wave + j (j = 0..4), column shifts 0..3
        u32x4_t fd[5][4];
        const uint16_t *hal = sD + ch * H_ELEMS;
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int hp = (2 * wave + j) * DS_HW + c + frow;
                fd[j][c] = *reinterpret_cast<const u32x4_t *>(hal + hp * BK + ((fsl ^ ds_swz(hp)) << 3));
            }
        const uint16_t *fil = sF + ch * F_ELEMS + foff;
        // output row 2p + a takes tap r when a + PAD - r is even, from dy row p + (a + PAD - r) / 2:
        // halo row index (p - p0 + 1) + (a + PAD - r) / 2
#pragma unroll
        for (int r = 0; r < DS_R; ++r)
#pragma unroll
            for (int s = 0; s < DS_R; ++s) {
                const int a = (r + DS_PAD) & 1, b = (s + DS_PAD) & 1;
                const int dr = (a + DS_PAD - r) / 2 + 1, dc = (b + DS_PAD - s) / 2 + 1;      // 0 .. 3
                const u32x4_t fw = *reinterpret_cast<const u32x4_t *>(fil + (r * DS_R + s) * 16 * BK);
#pragma unroll
                for (int i = 0; i < 2; ++i) acc[a][b][i] = T::mfma16(fw, fd[i + dr][dc], acc[a][b][i]);
            }
    }

    // ---- assemble the 32 x 32 x 16 output tile in LDS, write 1 KB rows -----------------
    __syncthreads();                                     // everyone has finished reading the operands
    uint16_t *const stg = lds;                           // [32 rows][32 pixels][16 channels]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const floatx4_t &c = acc[a][b][i];
                u32x2_t pk;
                pk[0] = (uint32_t)T::from_float(c[0]) | ((uint32_t)T::from_float(c[1]) << 16);
                pk[1] = (uint32_t)T::from_float(c[2]) | ((uint32_t)T::from_float(c[3]) << 16);
                const int row = 2 * (2 * wave + i) + a, col = 2 * frow + b;
                *reinterpret_cast<u32x2_t *>(stg + (row * 32 + col) * 16 + 4 * fsl) = pk;
            }
    __syncthreads();
    const int h0 = 2 * p0, w0 = 2 * q0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = wave * 4 + it, col = lane >> 1, c8 = (lane & 1) * 8;
        const int h = h0 + row, w = w0 + col;
        if (h >= p.H || w >= p.W || c8 >= p.C) continue;
        const u32x4_t v4 = *reinterpret_cast<const u32x4_t *>(stg + (row * 32 + col) * 16 + c8);
        *reinterpret_cast<u32x4_t *>(p.dx + ((size_t)(img * p.H + h) * p.W + w) * p.C + c8) = v4;
    }
}

bool dgrad_stem_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw)
{
    static const int mode = tuning_knob("DLCONV_DGRAD_STEM", 1); // tuning override: 0 = never
    (void)N;
    return mode && R == DS_R && S == DS_R && sh == 2 && sw == 2 && ph == DS_PAD && pw == DS_PAD && dh == 1 && dw == 1 &&
           (C == 8 || C == 16) && K % 8 == 0 && K <= DS_MAXCH * BK && H >= 2 && W >= 2;
}

size_t dgrad_stem_filter_bytes(int C, int K) { return (size_t)((K + BK - 1) / BK) * DS_R * DS_R * C * BK * sizeof(uint16_t); }

hipError_t launch_dgrad_stem(const DgradStemArgs &a, bool is_bf16, hipStream_t stream)
{
    const int PH = (a.H + 1) / 2, PW = (a.W + 1) / 2;
    const int64_t tiles = (int64_t)a.N * ((PH + DS_TP - 1) / DS_TP) * ((PW + DS_TP - 1) / DS_TP);
    if (tiles <= 0 || tiles > 0x7fffffff || a.K > DS_MAXCH * BK || a.C > 16) return hipErrorInvalidValue;
    // the forward output extent of such a layer: every dy pixel the halo addresses is bounded by it
    if (a.P != (a.H - 1) / 2 + 1 || a.Q != (a.W - 1) / 2 + 1) return hipErrorInvalidValue;
    if (is_bf16) DLK_LAUNCH("dgrad_stem_kernel", dgrad_stem_kernel<BF16>, dim3((unsigned)tiles), dim3(512), 0, stream, a);
    else DLK_LAUNCH("dgrad_stem_kernel", dgrad_stem_kernel<F16>, dim3((unsigned)tiles), dim3(512), 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
