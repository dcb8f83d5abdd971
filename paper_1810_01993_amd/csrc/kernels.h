// Host-visible launch interface of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <cstdio>
#include <string>
#ifdef DLCONV_TUNING
#include <cstdlib>
#endif

namespace dlk {

// Launch log.  dl_conv_describe() answers "which kernels would this call launch?" by walking the
// very code of the entry point with this pointer set: every launch then appends its kernel's name
// and grid to the log INSTEAD of launching, so the answer cannot drift from the dispatch.  The
// pointer is thread-local and non-null only inside that query.
struct LaunchLog { std::string text; };
extern thread_local LaunchLog *launch_log;
inline bool log_launch(const std::string &label, const dim3 &grid)
{
    if (!launch_log) return false;
    char g[48];
    if (grid.y > 1 || grid.z > 1) std::snprintf(g, sizeof g, "[%ux%ux%u]", grid.x, grid.y, grid.z);
    else std::snprintf(g, sizeof g, "[%u]", grid.x);
    if (!launch_log->text.empty()) launch_log->text += "; ";
    launch_log->text += label + g;
    return true;
}
// What a launch function returns after its launches: the runtime's verdict, or success while logging.
inline hipError_t launch_status() { return launch_log ? hipSuccess : hipGetLastError(); }
inline std::string kname(const char *base, std::initializer_list<int> params)
{
    std::string s = std::string(base) + "<";
    bool first = true;
    for (int v : params) { s += (first ? "" : ",") + std::to_string(v); first = false; }
    return s + ">";
}
#define DLK_LAUNCH(label, kernel, grid, block, lds, stream, ...)                                       \
    do {                                                                                               \
        if (!dlk::log_launch(label, dim3(grid))) hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__); \
    } while (0)

// Sweep knobs.  The library as shipped has none: which kernel runs, with which tiles and in which
// summation order, depends on the arguments of the call alone and never on the caller's
// environment.  Only a build made with -DDLCONV_TUNING (kernel sweeps) reads the named variable.
#ifdef DLCONV_TUNING
inline int tuning_knob(const char *name, int dflt)
{
    const char *e = std::getenv(name);
    return e ? std::atoi(e) : dflt;
}
#else
constexpr int tuning_knob(const char *, int dflt) { return dflt; }
#endif

// Implicit-GEMM convolution engine: D[m, j] = sum_{t, c} A[pixel(m, t), c] * B[j, t, c].
//   m indexes (n, oh, ow) of an output grid [N, OH, OW]; t = (jr, js) a grid of
//   TR x TS taps; the input pixel of tap t is
//       ih = oh*sh + th0 + jr*dth,   iw = ow*sw + tw0 + js*dtw,
//   outside [0,IH) x [0,IW) it contributes zero.  B is [Nout][TR*TS*Cin],
//   reduction index contiguous.  Row m is stored at
//       D + (((n*FH) + oh*osh + ooh)*FW + ow*osw + oow)*ldd.
// The forward pass uses it directly; the data gradient uses it once per
// stride-parity class of the input pixels with a re-laid-out filter.
struct IgemmArgs {
    const uint16_t *A;
    const uint16_t *B;
    uint16_t *D;
    int32_t NB;                 // batch
    int32_t IH, IW, Cin;        // A extents
    int32_t OH, OW;             // output grid of this launch
    int32_t Nout;               // GEMM N
    int32_t TR, TS;             // tap grid
    int32_t sh, sw;
    int32_t th0, dth, tw0, dtw;
    int32_t FH, FW, osh, osw, ooh, oow, ldd;
    int32_t c_outer;            // direct-to-LDS engine only: channel-major reduction order
    // Split reduction (direct-to-LDS engine, channel-major order, dense output with ldd == Nout):
    // with ksplits > 1 the 32-channel chunks are cut into ksplits ranges of split_chunks chunks,
    // range z (grid.y) writes fp32 partial sums to part[z][m][j] and an ordered reduce follows.
    int32_t ksplits, split_chunks;
    float *part;                // scratch for the partial sums, or null: never split
    // Filter given reduction-major (direct-to-LDS engine, channel-major order, Nout % 8 == 0): with
    // b_transposed != 0 element (column j, tap (jr, js), reduction channel c) of the filter operand is
    // B[b_base + j + jr*b_sr + js*b_ss + c*b_ldk], i.e. contiguous along the columns -- how the data
    // gradient finds it in the [K][R][S][C] filter.  Tiles are then deposited [channel][column] and the
    // fragments come from LDS transpose reads, so no re-laid-out copy is needed.
    int32_t b_transposed;
    int32_t b_base, b_sr, b_ss, b_ldk;
    int32_t b_elems;            // elements of the tensor B points into (bounds of the loads)
    // Point-wise tail fused into the store: D = act(sum + bias[column]).  bias: fp32, one value per
    // output column of THIS launch (null: none); relu != 0: negative results become zero.
    const float *bias;
    int32_t relu;
    // ... + resid[same element as D] before the activation (the skip connection of a residual block):
    // indexed exactly like D (a launch that offsets D by columns offsets resid alike); null: none.
    // The kernels with an LDS-staged coalesced store that cannot reach it before rounding (3x3 halo-tile,
    // narrow / wide 5x5) do not take such launches; the plain engine, the general halo-tile kernel, the
    // streaming kernel for few input channels and the split reduction do.
    const uint16_t *resid;
};

// Up to four GEMMs for one launch of the direct-to-LDS engine (see igemm_dma_batch_kernel).
struct IgemmBatch {
    static constexpr int MAX = 4;
    IgemmArgs a[MAX];
    int32_t n;
};

// Tile configuration (as for launch_igemm_dma) if these n GEMMs can share one launch of the
// direct-to-LDS engine, or -1: all must take the same configuration of the plain engine in
// channel-major order, unsplit, with the filter given the same way.
int igemm_batch_cfg(const IgemmArgs *a, int n);
hipError_t launch_igemm_batch(const IgemmBatch &b, bool is_bf16, hipStream_t stream);
hipError_t launch_igemm_dma_batch(const IgemmBatch &b, bool is_bf16, int cfg, hipStream_t stream);

// Would launch_igemm accept this GEMM with a reduction-major filter (b_transposed)?
bool igemm_accepts_transposed_b(const IgemmArgs &a);

// Bytes of partial-sum scratch launch_igemm would use for this GEMM if a.part were set (0: it would not split).
size_t igemm_split_bytes(const IgemmArgs &a);

// is_bf16 selects the MFMA flavour and the output rounding.
hipError_t launch_igemm(const IgemmArgs &a, bool is_bf16, hipStream_t stream);

// Direct-to-LDS variant of the engine (needs Cin % 8 == 0); cfg selects the tile.
hipError_t launch_igemm_dma(const IgemmArgs &a, bool is_bf16, int cfg, hipStream_t stream);

// Halo-tile variant for stride-1 multi-tap filters.  a.B must point at the
// blocked filter copy [chunk][tap][a.Nout][32] made by launch_filter_block.
int igemm_halo_columns(const IgemmArgs &a);
// Dense 5x5, unit stride and dilation, forward-oriented taps, 8..32 output columns (a multiple of 8), D 16-byte
// aligned: one 32-wide column tile per 16 x 32 pixel patch; a.B as for the other halo-tile kernels.
bool igemm_narrow5x5_applicable(const IgemmArgs &a);
// fp32 scratch (a.part) the launch needs when it splits the reduction (maps with few patches), else 0
size_t igemm_narrow5x5_split_bytes(const IgemmArgs &a);
hipError_t launch_igemm_narrow5x5(const IgemmArgs &a, bool is_bf16, hipStream_t stream);
// The mirror case: dense 5x5, unit stride and dilation, taps forward or mirrored, at most 32 input channels (one
// chunk), more than 32 output columns (a multiple of 4), D 8-byte aligned: the data gradient of such a layer.
bool igemm_wide5x5_applicable(const IgemmArgs &a);
hipError_t launch_igemm_wide5x5(const IgemmArgs &a, bool is_bf16, hipStream_t stream);
bool igemm_halo3x3_applicable(const IgemmArgs &a);
int64_t igemm_halo3x3_tiles(const IgemmArgs &a);
hipError_t launch_igemm_halo3x3(const IgemmArgs &a, bool is_bf16, hipStream_t stream);
size_t igemm_blocked_filter_bytes(const IgemmArgs &a);
hipError_t launch_igemm_halo(const IgemmArgs &a, bool is_bf16, hipStream_t stream);

// dst[((chunk*TR*TS + jr*TS + js)*Nrows + j)*32 + e] = src[base + j*sj + jr*sr + js*ss + (chunk*32+e)*sc],
// zero where chunk*32 + e >= Cin.
struct FilterBlockArgs {
    const uint16_t *src;
    uint16_t *dst;
    int64_t base, sj, sr, ss, sc;
    int32_t Nrows, TR, TS, Cin;
};
hipError_t launch_filter_block(const FilterBlockArgs &a, hipStream_t stream);

// Data gradient of a 7x7, stride-2, padding-3 convolution with 8 or 16 input channels and at most
// 64 output channels (the stem): all four parity classes in one workgroup, operands resident in LDS.
// wblk: the filter as [chunk of K][tap][c][32] (launch_filter_block with rows = c).
struct DgradStemArgs {
    const uint16_t *dy;         // [N][P][Q][K]
    const uint16_t *wblk;
    uint16_t *dx;               // [N][H][W][C]
    int32_t N, H, W, C, K, P, Q;
};
bool dgrad_stem_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw);
size_t dgrad_stem_filter_bytes(int C, int K);
hipError_t launch_dgrad_stem(const DgradStemArgs &a, bool is_bf16, hipStream_t stream);

// Filter re-layout for the data gradient: for one stride-parity class,
//   wt[c][jr][js][k] = w[k][r0 + jr*rstep][s0 + js*sstep][c]
struct FilterRelayoutArgs {
    const uint16_t *w;          // [K][R][S][C]
    uint16_t *wt;               // [C][TR][TS][K]
    int32_t K, R, S, C;
    int32_t r0, rstep, TR, s0, sstep, TS;
};
hipError_t launch_filter_relayout(const FilterRelayoutArgs &a, hipStream_t stream);
// Clears the pixels of dx[N][H][W][C] (C % 8 == 0, sh * sw <= 64) whose stride-parity class (h % sh) * sw + (w % sw)
// has its bit set in `mask`.
hipError_t launch_zero_classes(uint16_t *dx, int N, int H, int W, int C, int sh, int sw, uint64_t mask, hipStream_t stream);

// Filter gradient: partial[z][k][j] = sum over the z-th slice of the N*P*Q
// pixels of dy[pix][k] * x[pixel(pix, tap(j)), c(j)],  j = (r*S + s)*C + c.
struct WgradArgs {
    const uint16_t *x;          // [N,H,W,C]
    const uint16_t *dy;         // [N,P,Q,K]
    float *partial;             // [splits][K][R*S*C]
    int32_t N, H, W, C, K, R, S, P, Q;
    int32_t sh, sw, ph, pw, dh, dw;
    int32_t splits;             // slices of the pixel range
    int32_t chunk;              // pixels per slice, multiple of 32
    int32_t spread;             // direct-to-LDS kernel: deal the tiles of a slice over all XCDs (few slices)
};
hipError_t launch_wgrad(const WgradArgs &a, bool is_bf16, hipStream_t stream);

// Direct-to-LDS variant (needs K % 8 == 0 and C % 8 == 0); cfg selects the tile.
hipError_t launch_wgrad_dma(const WgradArgs &a, bool is_bf16, int cfg, hipStream_t stream);

// Kernel choice and reduction split for one filter gradient, shared by the
// workspace query and the launch.  cfg < 0: register-staged kernel.
struct WgradPlan {
    int cfg;
    int splits;
    int chunk;                  // pixels per slice, multiple of 32
    int spread;                 // see WgradArgs
};
WgradPlan wgrad_make_plan(int64_t npix, int K, int C, int RSC, bool thin_ok);

// Filter gradient of dense RxR (3x3 or 5x5), stride 1, dilation 1, "same"-padded layers on large images by
// the strip-walk kernels (cfg -3 / -4 of the plan): all taps per workgroup, partial[slice][K][R*R][C].
struct WgradStripArgs {
    const uint16_t *x;          // [N,H,W,C]
    const uint16_t *dy;         // [N,H,W,K]
    float *partial;             // [slices][K][R][R][C]
    int32_t N, H, W, C, K;
    int32_t slices;             // N * ceil(H / rs) * ceil(ceil(W / 32) / xs)
    int32_t rs, xs;             // image rows and 32-pixel strips per slice
};
struct WgradStripPlan { int slices, rs, xs; };
bool wgrad3x3_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw);
WgradStripPlan wgrad3x3_make_plan(int N, int H, int W, int C, int K);
hipError_t launch_wgrad3x3(const WgradStripArgs &a, bool is_bf16, hipStream_t stream);
// The same for dense 5x5, stride 1, padding 2 with at most 32 output channels (same argument and plan structs;
// partial sums [slice][K][5][5][C]).
bool wgrad5x5_applicable(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int dh, int dw);
WgradStripPlan wgrad5x5_make_plan(int N, int H, int W, int C, int K);
hipError_t launch_wgrad5x5(const WgradStripArgs &a, bool is_bf16, hipStream_t stream);

// Streaming kernels for 1x1 layers with <= 4 channels on one side (cfg -2 of the plan).
bool thin_rows_applicable(const IgemmArgs &a);
hipError_t launch_thin_rows(const IgemmArgs &a, bool is_bf16, hipStream_t stream);
bool thin_cols_applicable(const IgemmArgs &a);
hipError_t launch_thin_cols(const IgemmArgs &a, bool is_bf16, hipStream_t stream);
bool thin_wgrad_applicable(int K, int C, int R, int S, int sh, int sw, int ph, int pw);
hipError_t launch_thin_wgrad(const WgradArgs &a, bool is_bf16, hipStream_t stream);

// dw[i] = sum_z partial[z][i] in ascending z, rounded to out_dtype (dl_dtype).
hipError_t launch_splitk_reduce(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype,
                                hipStream_t stream);
// The same with the forward convolution's point-wise tail: element i belongs to column i % ncols.
hipError_t launch_splitk_reduce_tail(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype,
                                     const float *bias, int32_t relu, int32_t ncols, const uint16_t *resid, hipStream_t stream);

// Backward of the point-wise tail y = max(s + bias, 0): dz = dy masked by y > 0 (relu != 0;
// otherwise dz and y are not touched), dbias = column sums of dz.  partial: blocks x K floats.
struct TailBwdArgs {
    const uint16_t *dy, *y;     // [npix][K]
    uint16_t *dz;
    float *partial, *dbias;
    int64_t npix, chunk;        // chunk: pixels per workgroup (set by the launcher)
    int32_t K, relu;
};
int tail_bwd_blocks(int64_t npix, int K);
hipError_t launch_tail_bwd(const TailBwdArgs &a, bool is_bf16, hipStream_t stream);

// LARC update of up to LARC_MAX tensors (see larc.hip).  partial: 2 * LARC_SLICES floats per tensor
// of the whole call; first: index of t[0] among the call's tensors; rates: per-tensor rate out, or null.
constexpr int LARC_MAX = 64, LARC_SLICES = 256;
struct LarcTensor { float *w; const void *g; float *v; int64_t count; };
struct LarcBatch {
    LarcTensor t[LARC_MAX];
    float *partial, *rates;
    float lr, trust, wd, momentum, eps;
    int32_t clip, n, first;
};
hipError_t launch_larc(const LarcBatch &b, int grad_dtype, hipStream_t stream);

// Weighted per-pixel cross-entropy, 3 classes.
int ce_num_blocks(int64_t n_pixels);
// The logits layer (1x1, C -> 3) fused with the loss: one pass over x.  C % 8 == 0, 32 <= C <= 2048.
struct LogitsCeArgs {
    const uint16_t *x;          // [n][C]
    const uint16_t *w;          // [3][C]
    const uint8_t *labels;      // [n]
    const float *cw;            // [3]
    float scale;
    int64_t n;
    int32_t C;
    uint16_t *logits;           // [n][3] or null
    uint16_t *dlogits;          // [n][3] or null
    uint16_t *dx;               // [n][C]
    float *partial_dw;          // [blocks][3][C]
    float *partial_loss;        // [blocks]
};
int logits_ce_blocks(int64_t n_pixels, int C);
hipError_t launch_logits_ce(const LogitsCeArgs &a, bool is_bf16, hipStream_t stream);
// loss[0] = scale * (sum of the partials, in a fixed order)
hipError_t ce_static_partials(float **ptr);      // library-owned partial sums (per device) for the call without a workspace
hipError_t launch_ce_finish(const float *partials, int n_partials, float scale, float *loss, hipStream_t stream);
hipError_t launch_weighted_ce(const uint16_t *logits, bool is_bf16, const uint8_t *labels, const float *weights,
                              bool per_pixel, float scale, int64_t n_pixels, float *loss, uint16_t *dlogits,
                              float *partials, hipStream_t stream);


}  // namespace dlk
