// C boundary: argument validation, workspace sizing, and the mapping of the
// three convolution passes and the loss onto the gfx950 kernels.  Everything
// here runs on the host; validation happens before any launch.
#include <algorithm>
#include <hip/hip_runtime.h>

#include "../../include/dlconv.h"
#include "kernels.h"

namespace dlk {
thread_local LaunchLog *launch_log = nullptr;
}

namespace {

constexpr int64_t MAX_ELEMS = 0x7FF00000;     // 32-bit byte offsets, with room above for the out-of-range marker

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int gcd(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

struct Geometry {
    int32_t P, Q;
    int64_t x_elems, w_elems, y_elems;
};

dl_status check_desc(const dl_conv_desc *d, Geometry *g)
{
    if (!d) return DL_ERR_NULL;
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->K < 1 || d->R < 1 || d->S < 1) return DL_ERR_SHAPE;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return DL_ERR_SHAPE;
    if (d->dtype != DL_F16 && d->dtype != DL_BF16) return DL_ERR_DTYPE;
    if (d->dw_dtype != d->dtype && d->dw_dtype != DL_F32) return DL_ERR_DTYPE;
    const int64_t span_h = (int64_t)d->H + 2 * (int64_t)d->pad_h - (int64_t)d->dil_h * (d->R - 1) - 1;
    const int64_t span_w = (int64_t)d->W + 2 * (int64_t)d->pad_w - (int64_t)d->dil_w * (d->S - 1) - 1;
    if (span_h < 0 || span_w < 0) return DL_ERR_SHAPE;
    const int64_t P = span_h / d->stride_h + 1, Q = span_w / d->stride_w + 1;
    // padded coordinates and tensor sizes must fit the kernels' 32-bit index math
    if ((int64_t)d->H + 2 * (int64_t)d->pad_h >= MAX_ELEMS || (int64_t)d->W + 2 * (int64_t)d->pad_w >= MAX_ELEMS)
        return DL_ERR_SHAPE;
    const int64_t xe = (int64_t)d->N * d->H * d->W;
    const int64_t ye = (int64_t)d->N * P * Q;
    const int64_t we = (int64_t)d->R * d->S * d->C;
    if (xe >= MAX_ELEMS || ye >= MAX_ELEMS || we >= MAX_ELEMS) return DL_ERR_SHAPE;
    if (xe * d->C >= MAX_ELEMS || ye * d->K >= MAX_ELEMS || we * d->K >= MAX_ELEMS) return DL_ERR_SHAPE;
    g->P = (int32_t)P;
    g->Q = (int32_t)Q;
    g->x_elems = xe * d->C;
    g->y_elems = ye * d->K;
    g->w_elems = we * d->K;
    return DL_OK;
}

// Taps of one axis that reach input positions congruent to `a` modulo the
// stride: r = r0 + j*rstep, j < count, and the output position they read is
// (pos/stride-class index) + t0 + j*dt.
struct AxisTaps { int r0, rstep, count, t0, dt; };

AxisTaps class_taps(int a, int R, int stride, int pad, int dil)
{
    AxisTaps t{0, 1, 0, 0, 0};
    t.rstep = stride / gcd(dil, stride);
    int r0 = -1;
    for (int r = 0; r < R && r < t.rstep; ++r)
        if (((a + pad - r * dil) % stride + stride) % stride == 0) { r0 = r; break; }
    if (r0 < 0) return t;                               // no tap reaches this class
    t.r0 = r0;
    t.count = (R - 1 - r0) / t.rstep + 1;
    t.t0 = (a + pad - r0 * dil) / stride;               // exact by construction
    t.dt = -(t.rstep * dil) / stride;                   // exact: rstep*dil is a multiple of stride
    return t;
}

// ---- one implicit GEMM, with the halo-tile kernel where it applies ------------
// Where the coefficients of the GEMM's filter operand live in the caller's
// filter tensor: element (row j, tap (jr, js), reduction channel c) is
// src[base + j*sj + jr*sr + js*ss + c*sc].
struct FilterSrc { const uint16_t *src; int64_t base, sj, sr, ss, sc; };

int halo_columns(const dlk::IgemmArgs &a) { return dlk::igemm_halo_columns(a); }

// Scratch one implicit GEMM needs: the blocked filter copy of a halo kernel, or the fp32 partial
// sums of a split reduction of the plain engine (never both).
size_t igemm_scratch_bytes(const dlk::IgemmArgs &a)
{
    const int cols = halo_columns(a);
    if (!cols) return align_up(dlk::igemm_split_bytes(a), 256);
    dlk::IgemmArgs h = a;
    h.Nout = cols;
    // (the 5x5 kernel for at most 32 output channels may split its reduction on small maps: partial sums behind the copy)
    const size_t part = dlk::igemm_narrow5x5_applicable(h) ? align_up(dlk::igemm_narrow5x5_split_bytes(h), 256) : 0;
    return align_up(dlk::igemm_blocked_filter_bytes(h), 256) + part;
}

// a.B: plain [Nout][taps*Cin] filter (may be null if the halo kernel takes every column).
hipError_t run_igemm(const dlk::IgemmArgs &a, bool bf16, const FilterSrc &fs, uint16_t *scratch, hipStream_t stream)
{
    const int cols = halo_columns(a);
    if (!cols) {
        dlk::IgemmArgs g = a;
        g.part = dlk::igemm_split_bytes(a) ? reinterpret_cast<float *>(scratch) : nullptr;
        return dlk::launch_igemm(g, bf16, stream);
    }
    dlk::FilterBlockArgs f{};
    f.src = fs.src; f.dst = scratch;
    f.base = fs.base; f.sj = fs.sj; f.sr = fs.sr; f.ss = fs.ss; f.sc = fs.sc;
    f.Nrows = cols; f.TR = a.TR; f.TS = a.TS; f.Cin = a.Cin;
    hipError_t e = dlk::launch_filter_block(f, stream);
    if (e != hipSuccess) return e;
    dlk::IgemmArgs h = a;
    h.Nout = cols;
    h.B = scratch;
    h.part = reinterpret_cast<float *>(reinterpret_cast<char *>(scratch) + align_up(dlk::igemm_blocked_filter_bytes(h), 256));
    e = dlk::launch_igemm_halo(h, bf16, stream);
    if (e != hipSuccess || cols == a.Nout) return e;
    dlk::IgemmArgs r = a;
    r.Nout = a.Nout - cols;
    r.B = a.B + (size_t)cols * a.TR * a.TS * a.Cin;
    r.D = a.D + cols;
    if (a.bias) r.bias = a.bias + cols;
    if (a.resid) r.resid = a.resid + cols;
    return dlk::launch_igemm(r, bf16, stream);
}

dlk::IgemmArgs fwd_args(const dl_conv_desc *d, const Geometry &g)
{
    dlk::IgemmArgs a{};
    a.NB = d->N; a.IH = d->H; a.IW = d->W; a.Cin = d->C;
    a.OH = g.P; a.OW = g.Q; a.Nout = d->K;
    a.TR = d->R; a.TS = d->S;
    a.sh = d->stride_h; a.sw = d->stride_w;
    a.th0 = -d->pad_h; a.dth = d->dil_h; a.tw0 = -d->pad_w; a.dtw = d->dil_w;
    a.FH = g.P; a.FW = g.Q; a.osh = 1; a.osw = 1; a.ooh = 0; a.oow = 0; a.ldd = d->K;
    return a;
}

// The data gradient of one stride-parity class (ca, cb) of the input pixels.
struct DgradClass {
    dlk::IgemmArgs args;        // pointers unset
    AxisTaps th, tw;
    bool empty, has_taps;
    size_t wt_bytes, blk_bytes;
};

DgradClass dgrad_class(const dl_conv_desc *d, const Geometry &g, int ca, int cb)
{
    DgradClass c{};
    const int OH = ca < d->H ? (d->H - ca + d->stride_h - 1) / d->stride_h : 0;
    const int OW = cb < d->W ? (d->W - cb + d->stride_w - 1) / d->stride_w : 0;
    c.th = class_taps(ca, d->R, d->stride_h, d->pad_h, d->dil_h);
    c.tw = class_taps(cb, d->S, d->stride_w, d->pad_w, d->dil_w);
    c.empty = OH == 0 || OW == 0;
    c.has_taps = c.th.count > 0 && c.tw.count > 0;
    c.wt_bytes = align_up((size_t)d->C * c.th.count * c.tw.count * d->K * sizeof(uint16_t), 256);
    dlk::IgemmArgs &a = c.args;
    a.NB = d->N; a.IH = g.P; a.IW = g.Q; a.Cin = d->K;
    a.OH = OH; a.OW = OW; a.Nout = d->C;
    a.TR = c.has_taps ? c.th.count : 0; a.TS = c.has_taps ? c.tw.count : 1;
    a.sh = 1; a.sw = 1;
    a.th0 = c.th.t0; a.dth = c.th.dt; a.tw0 = c.tw.t0; a.dtw = c.tw.dt;
    a.FH = d->H; a.FW = d->W; a.osh = d->stride_h; a.osw = d->stride_w; a.ooh = ca; a.oow = cb;
    a.ldd = d->C;
    c.blk_bytes = (c.empty || !c.has_taps) ? 0 : igemm_scratch_bytes(a);
    return c;
}

bool use_dgrad_stem(const dl_conv_desc *d)
{
    return dlk::dgrad_stem_applicable(d->N, d->H, d->W, d->C, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w,
                                      d->dil_h, d->dil_w);
}

size_t dgrad_workspace(const dl_conv_desc *d, const Geometry &g)
{
    if (use_dgrad_stem(d)) return align_up(dlk::dgrad_stem_filter_bytes(d->C, d->K), 256);
    size_t total = 0;
    for (int ca = 0; ca < d->stride_h; ++ca)
        for (int cb = 0; cb < d->stride_w; ++cb) {
            const DgradClass c = dgrad_class(d, g, ca, cb);
            total += c.wt_bytes + c.blk_bytes;
        }
    return total;
}

bool use_wgrad3x3(const dl_conv_desc *d)
{
    return dlk::wgrad3x3_applicable(d->N, d->H, d->W, d->C, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w,
                                    d->dil_h, d->dil_w);
}

bool use_wgrad5x5(const dl_conv_desc *d)
{
    return dlk::wgrad5x5_applicable(d->N, d->H, d->W, d->C, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w,
                                    d->dil_h, d->dil_w);
}

dlk::WgradPlan wgrad_plan(const dl_conv_desc *d, const Geometry &g)
{
    if (use_wgrad5x5(d)) {
        const dlk::WgradStripPlan p5 = dlk::wgrad5x5_make_plan(d->N, d->H, d->W, d->C, d->K);
        return dlk::WgradPlan{-4, p5.slices, 0};
    }
    if (use_wgrad3x3(d)) {
        const dlk::WgradStripPlan p3 = dlk::wgrad3x3_make_plan(d->N, d->H, d->W, d->C, d->K);
        return dlk::WgradPlan{-3, p3.slices, 0};
    }
    const bool thin = dlk::thin_wgrad_applicable(d->K, d->C, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w);
    return dlk::wgrad_make_plan((int64_t)d->N * g.P * g.Q, d->K, d->C, d->R * d->S * d->C, thin);
}

size_t wgrad_workspace(const dl_conv_desc *d, const Geometry &g)
{
    return (size_t)wgrad_plan(d, g).splits * (size_t)g.w_elems * sizeof(float);
}

dl_status hip_status(hipError_t e) { return e == hipSuccess ? DL_OK : DL_ERR_LAUNCH; }

}  // namespace

extern "C" {

dl_status dl_logits_ce_workspace_bytes(int64_t n_pixels, int32_t C, size_t *bytes)
{
    if (!bytes) return DL_ERR_NULL;
    if (n_pixels < 0 || C < 32 || C > 2048 || C % 8 != 0) return DL_ERR_SHAPE;
    const size_t blocks = (size_t)dlk::logits_ce_blocks(n_pixels, C);
    *bytes = align_up(blocks * 3 * (size_t)C * sizeof(float), 256) + align_up(blocks * sizeof(float), 256);
    return DL_OK;
}

dl_status logits_ce_fused_fwd_bwd(const void *x, const void *w, int32_t dtype, const uint8_t *labels,
                                  const float *class_weights, float scale, int64_t n_pixels, int32_t C, void *logits,
                                  float *loss, void *dlogits, void *dx, void *dw, int32_t dw_dtype, void *workspace,
                                  size_t workspace_bytes, void *hip_stream)
{
    if (!w || !class_weights || !loss || !dw) return DL_ERR_NULL;
    if (n_pixels < 0 || C < 32 || C > 2048 || C % 8 != 0 || n_pixels >= MAX_ELEMS / C) return DL_ERR_SHAPE;
    if (n_pixels > 0 && (!x || !labels || !dx)) return DL_ERR_NULL;
    if ((dtype != DL_F16 && dtype != DL_BF16) || (dw_dtype != dtype && dw_dtype != DL_F32)) return DL_ERR_DTYPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(dx) || !aligned16(dw)) return DL_ERR_ALIGN;
    size_t need = 0;
    dl_logits_ce_workspace_bytes(n_pixels, C, &need);
    if (!workspace || workspace_bytes < need) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int blocks = dlk::logits_ce_blocks(n_pixels, C);
    dlk::LogitsCeArgs a{};
    a.x = static_cast<const uint16_t *>(x);
    a.w = static_cast<const uint16_t *>(w);
    a.labels = labels;
    a.cw = class_weights;
    a.scale = scale;
    a.n = n_pixels;
    a.C = C;
    a.logits = static_cast<uint16_t *>(logits);
    a.dlogits = static_cast<uint16_t *>(dlogits);
    a.dx = static_cast<uint16_t *>(dx);
    a.partial_dw = static_cast<float *>(workspace);
    a.partial_loss = reinterpret_cast<float *>(static_cast<char *>(workspace) + align_up((size_t)blocks * 3 * C * sizeof(float), 256));
    if (dlk::launch_logits_ce(a, dtype == DL_BF16, stream) != hipSuccess) return DL_ERR_LAUNCH;
    if (dlk::launch_splitk_reduce(a.partial_dw, blocks, (int64_t)3 * C, dw, dw_dtype, stream) != hipSuccess) return DL_ERR_LAUNCH;
    return hip_status(dlk::launch_ce_finish(a.partial_loss, blocks, scale, loss, stream));
}

const char *dl_status_string(dl_status s)
{
    switch (s) {
        case DL_OK: return "ok";
        case DL_ERR_NULL: return "null pointer";
        case DL_ERR_SHAPE: return "invalid shape";
        case DL_ERR_DTYPE: return "unsupported dtype";
        case DL_ERR_ALIGN: return "tensor base not 16-byte aligned";
        case DL_ERR_WORKSPACE: return "workspace missing or too small";
        case DL_ERR_UNSUPPORTED: return "unsupported configuration";
        case DL_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

dl_status dl_conv_out_shape(const dl_conv_desc *desc, int32_t *P, int32_t *Q)
{
    if (!desc || !P || !Q) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(desc, &g);
    if (st != DL_OK) return st;
    *P = g.P;
    *Q = g.Q;
    return DL_OK;
}

dl_status dl_conv_workspace_bytes(const dl_conv_desc *desc, int pass, size_t *bytes)
{
    if (!desc || !bytes) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(desc, &g);
    if (st != DL_OK) return st;
    switch (pass) {
        case DL_PASS_FWD: {
            // with a residual input some kernels are not available and the choice of scratch changes: enough for either
            dlk::IgemmArgs a = fwd_args(desc, g);
            const size_t plain = igemm_scratch_bytes(a);
            a.resid = reinterpret_cast<const uint16_t *>(uintptr_t(16));     // any non-null value: only tested for null
            *bytes = std::max(plain, igemm_scratch_bytes(a));
            return DL_OK;
        }
        case DL_PASS_BWD_DATA: *bytes = dgrad_workspace(desc, g); return DL_OK;
        case DL_PASS_BWD_FILTER: *bytes = wgrad_workspace(desc, g); return DL_OK;
    }
    return DL_ERR_UNSUPPORTED;
}

namespace {
dl_status run_fwd(const dl_conv_desc *d, const void *x, const void *w, const float *bias, const void *residual, int relu,
                  void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !x || !w || !y) return DL_ERR_NULL;
    if (residual && !aligned16(residual)) return DL_ERR_ALIGN;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return DL_ERR_ALIGN;
    if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)) return DL_ERR_ALIGN;
    dlk::IgemmArgs a = fwd_args(d, g);
    a.resid = static_cast<const uint16_t *>(residual);    // decides which kernels may take the launch
    const size_t need = igemm_scratch_bytes(a);
    if (need > 0 && (!workspace || workspace_bytes < need)) return DL_ERR_WORKSPACE;
    if (need > 0 && !aligned16(workspace)) return DL_ERR_ALIGN;
    a.A = static_cast<const uint16_t *>(x);
    a.B = static_cast<const uint16_t *>(w);
    a.D = static_cast<uint16_t *>(y);
    a.bias = bias;
    a.relu = relu ? 1 : 0;
    const FilterSrc fs{a.B, 0, (int64_t)d->R * d->S * d->C, (int64_t)d->S * d->C, d->C, 1};
    return hip_status(run_igemm(a, d->dtype == DL_BF16, fs, static_cast<uint16_t *>(workspace),
                                static_cast<hipStream_t>(hip_stream)));
}
}  // namespace

dl_status conv2d_fwd(const dl_conv_desc *d, const void *x, const void *w, void *y, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    return run_fwd(d, x, w, nullptr, nullptr, 0, y, workspace, workspace_bytes, hip_stream);
}

dl_status conv2d_fwd_bias_relu(const dl_conv_desc *d, const void *x, const void *w, const float *bias, int32_t relu,
                               void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_fwd(d, x, w, bias, nullptr, relu, y, workspace, workspace_bytes, hip_stream);
}

dl_status conv2d_fwd_bias_add_relu(const dl_conv_desc *d, const void *x, const void *w, const float *bias,
                                   const void *residual, int32_t relu, void *y, void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    return run_fwd(d, x, w, bias, residual, relu, y, workspace, workspace_bytes, hip_stream);
}

dl_status conv2d_bwd_data(const dl_conv_desc *d, const void *dy, const void *w, void *dx, void *workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    if (!d || !dy || !w || !dx) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return DL_ERR_ALIGN;
    const size_t need = dgrad_workspace(d, g);
    if (need > 0 && (!workspace || workspace_bytes < need)) return DL_ERR_WORKSPACE;
    if (need > 0 && !aligned16(workspace)) return DL_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool bf16 = d->dtype == DL_BF16;

    if (use_dgrad_stem(d)) {
        // few input channels, 7x7 stride 2: all parity classes in one workgroup, operands resident in LDS
        dlk::FilterBlockArgs f{};
        f.src = static_cast<const uint16_t *>(w);
        f.dst = static_cast<uint16_t *>(workspace);
        f.base = 0; f.sj = 1; f.sr = (int64_t)d->S * d->C; f.ss = d->C; f.sc = (int64_t)d->R * d->S * d->C;
        f.Nrows = d->C; f.TR = d->R; f.TS = d->S; f.Cin = d->K;
        if (dlk::launch_filter_block(f, stream) != hipSuccess) return DL_ERR_LAUNCH;
        dlk::DgradStemArgs a{};
        a.dy = static_cast<const uint16_t *>(dy);
        a.wblk = f.dst;
        a.dx = static_cast<uint16_t *>(dx);
        a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.K = d->K; a.P = g.P; a.Q = g.Q;
        return hip_status(dlk::launch_dgrad_stem(a, bf16, stream));
    }

    // Input pixels (h, w) fall into stride_h*stride_w parity classes; within a
    // class the contributing taps and the output pixels they pair with form
    // regular grids, so each class is one dense implicit GEMM over dy with the
    // filter re-laid-out as [c][tap][k].  Classes that take the plain engine with
    // one tile shape share a launch (their tiles of one image region then run
    // side by side); the others are launched one by one.
    struct Pending { dlk::IgemmArgs a; FilterSrc fs; uint16_t *blk; };
    Pending pending[dlk::IgemmBatch::MAX];
    int n_pending = 0;
    bool overflow = false;
    size_t ws_off = 0;
    // classes that no tap reaches (e.g. three of the four of a 1x1 stride-2 layer) are all zeros: one fill for all
    uint64_t zero_mask = 0;
    if (d->C % 8 == 0 && d->stride_h * d->stride_w <= 64) {
        for (int ca = 0; ca < d->stride_h; ++ca)
            for (int cb = 0; cb < d->stride_w; ++cb) {
                const DgradClass c = dgrad_class(d, g, ca, cb);
                if (!c.empty && !c.has_taps) zero_mask |= 1ull << (ca * d->stride_w + cb);
            }
        if (zero_mask && dlk::launch_zero_classes(static_cast<uint16_t *>(dx), d->N, d->H, d->W, d->C, d->stride_h, d->stride_w,
                                                  zero_mask, stream) != hipSuccess)
            return DL_ERR_LAUNCH;
    }
    for (int ca = 0; ca < d->stride_h; ++ca)
        for (int cb = 0; cb < d->stride_w; ++cb) {
            DgradClass c = dgrad_class(d, g, ca, cb);
            uint16_t *wt = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) + ws_off);
            uint16_t *blk = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) + ws_off + c.wt_bytes);
            ws_off += c.wt_bytes + c.blk_bytes;
            if (c.empty || ((zero_mask >> (ca * d->stride_w + cb)) & 1)) continue;
            dlk::IgemmArgs &a = c.args;
            a.A = static_cast<const uint16_t *>(dy);
            a.D = static_cast<uint16_t *>(dx);
            a.B = static_cast<const uint16_t *>(w);     // never read when there are no taps
            const bool all_halo = c.has_taps && halo_columns(a) == a.Nout;
            const int64_t SC = (int64_t)d->S * d->C;
            // the plain engine can take the filter as it lies in memory (reduction-major for this GEMM)
            const bool direct = c.has_taps && halo_columns(a) == 0 && dlk::igemm_accepts_transposed_b(a);
            if (direct) {
                a.b_transposed = 1;
                a.b_base = (int32_t)(c.th.r0 * SC + (int64_t)c.tw.r0 * d->C);
                a.b_sr = (int32_t)(c.th.rstep * SC);
                a.b_ss = (int32_t)((int64_t)c.tw.rstep * d->C);
                a.b_ldk = (int32_t)((int64_t)d->R * SC);
                a.b_elems = (int32_t)g.w_elems;
            } else if (c.has_taps && !all_halo) {
                dlk::FilterRelayoutArgs f{};
                f.w = static_cast<const uint16_t *>(w);
                f.wt = wt;
                f.K = d->K; f.R = d->R; f.S = d->S; f.C = d->C;
                f.r0 = c.th.r0; f.rstep = c.th.rstep; f.TR = c.th.count;
                f.s0 = c.tw.r0; f.sstep = c.tw.rstep; f.TS = c.tw.count;
                if (dlk::launch_filter_relayout(f, stream) != hipSuccess) return DL_ERR_LAUNCH;
                a.B = wt;
            }
            const FilterSrc fs{static_cast<const uint16_t *>(w), c.th.r0 * SC + (int64_t)c.tw.r0 * d->C, 1,
                               c.th.rstep * SC, (int64_t)c.tw.rstep * d->C, (int64_t)d->R * SC};
            if (c.has_taps && halo_columns(a) == 0 && !overflow) {
                if (n_pending < dlk::IgemmBatch::MAX) {
                    pending[n_pending++] = Pending{a, fs, blk};
                    continue;
                }
                overflow = true;                        // more classes than one launch holds: one by one after all
            }
            if (run_igemm(a, bf16, fs, blk, stream) != hipSuccess) return DL_ERR_LAUNCH;
        }
    if (n_pending > 0) {
        dlk::IgemmBatch b{};
        b.n = n_pending;
        for (int i = 0; i < n_pending; ++i) b.a[i] = pending[i].a;
        if (!overflow && dlk::igemm_batch_cfg(b.a, b.n) >= 0) {
            if (dlk::launch_igemm_batch(b, bf16, stream) != hipSuccess) return DL_ERR_LAUNCH;
        } else {
            for (int i = 0; i < n_pending; ++i)
                if (run_igemm(pending[i].a, bf16, pending[i].fs, pending[i].blk, stream) != hipSuccess) return DL_ERR_LAUNCH;
        }
    }
    return DL_OK;
}

dl_status conv2d_bwd_filter(const dl_conv_desc *d, const void *x, const void *dy, void *dw, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    if (!d || !x || !dy || !dw) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw)) return DL_ERR_ALIGN;
    const dlk::WgradPlan plan = wgrad_plan(d, g);
    if (!workspace || workspace_bytes < wgrad_workspace(d, g)) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    dlk::WgradArgs a{};
    a.x = static_cast<const uint16_t *>(x);
    a.dy = static_cast<const uint16_t *>(dy);
    a.partial = static_cast<float *>(workspace);
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.K = d->K; a.R = d->R; a.S = d->S; a.P = g.P; a.Q = g.Q;
    a.sh = d->stride_h; a.sw = d->stride_w; a.ph = d->pad_h; a.pw = d->pad_w; a.dh = d->dil_h; a.dw = d->dil_w;
    a.splits = plan.splits;
    a.chunk = plan.chunk;
    a.spread = plan.spread;
    hipError_t e;
    if (plan.cfg == -3) {
        const dlk::WgradStripPlan p3 = dlk::wgrad3x3_make_plan(d->N, d->H, d->W, d->C, d->K);
        dlk::WgradStripArgs w{};
        w.x = a.x; w.dy = a.dy; w.partial = a.partial;
        w.N = d->N; w.H = d->H; w.W = d->W; w.C = d->C; w.K = d->K;
        w.slices = p3.slices; w.rs = p3.rs; w.xs = p3.xs;
        e = dlk::launch_wgrad3x3(w, d->dtype == DL_BF16, stream);
    } else if (plan.cfg == -4) {
        const dlk::WgradStripPlan p5 = dlk::wgrad5x5_make_plan(d->N, d->H, d->W, d->C, d->K);
        dlk::WgradStripArgs w{};
        w.x = a.x; w.dy = a.dy; w.partial = a.partial;
        w.N = d->N; w.H = d->H; w.W = d->W; w.C = d->C; w.K = d->K;
        w.slices = p5.slices; w.rs = p5.rs; w.xs = p5.xs;
        e = dlk::launch_wgrad5x5(w, d->dtype == DL_BF16, stream);
    } else
    e = plan.cfg >= 0    ? dlk::launch_wgrad_dma(a, d->dtype == DL_BF16, plan.cfg, stream)
                   : plan.cfg == -2 ? dlk::launch_thin_wgrad(a, d->dtype == DL_BF16, stream)
                                    : dlk::launch_wgrad(a, d->dtype == DL_BF16, stream);
    if (e != hipSuccess) return DL_ERR_LAUNCH;
    e = dlk::launch_splitk_reduce(a.partial, plan.splits, g.w_elems, dw, d->dw_dtype, stream);
    return hip_status(e);
}

dl_status dl_conv_describe(const dl_conv_desc *d, int pass, char *buf, size_t buf_bytes)
{
    if (!d || !buf) return DL_ERR_NULL;
    if (buf_bytes < 2) return DL_ERR_SHAPE;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (pass != DL_PASS_FWD && pass != DL_PASS_BWD_DATA && pass != DL_PASS_BWD_FILTER) return DL_ERR_UNSUPPORTED;
    // The entry point itself runs, on stand-in addresses that only pointer arithmetic ever touches,
    // with every launch turned into a log line.
    void *const a = reinterpret_cast<void *>(uintptr_t(1) << 40);
    void *const b = reinterpret_cast<void *>(uintptr_t(2) << 40);
    void *const c = reinterpret_cast<void *>(uintptr_t(3) << 40);
    void *const ws = reinterpret_cast<void *>(uintptr_t(4) << 40);
    size_t ws_bytes = 0;
    dl_conv_workspace_bytes(d, pass, &ws_bytes);
    dlk::LaunchLog log;
    dlk::launch_log = &log;
    dl_status r;
    if (pass == DL_PASS_FWD) r = conv2d_fwd(d, a, b, c, ws, ws_bytes, nullptr);
    else if (pass == DL_PASS_BWD_DATA) r = conv2d_bwd_data(d, a, b, c, ws, ws_bytes, nullptr);
    else r = conv2d_bwd_filter(d, a, b, c, ws, ws_bytes, nullptr);
    dlk::launch_log = nullptr;
    if (r != DL_OK) return r;
    const size_t n = log.text.size() < buf_bytes - 1 ? log.text.size() : buf_bytes - 1;
    log.text.copy(buf, n);
    buf[n] = 0;
    return DL_OK;
}

// The transposed convolution and its two gradients are the three passes of the underlying
// convolution with the operand roles exchanged: the layer's input stands where that
// convolution's output gradient stands, its output where the data gradient stands.
dl_status conv2d_transpose_fwd(const dl_conv_desc *d, const void *x, const void *w, void *y, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    return conv2d_bwd_data(d, x, w, y, workspace, workspace_bytes, hip_stream);
}

dl_status conv2d_transpose_bwd_data(const dl_conv_desc *d, const void *dy, const void *w, void *dx, void *workspace,
                                    size_t workspace_bytes, void *hip_stream)
{
    return conv2d_fwd(d, dy, w, dx, workspace, workspace_bytes, hip_stream);
}

dl_status conv2d_transpose_bwd_filter(const dl_conv_desc *d, const void *x, const void *dy, void *dw,
                                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return conv2d_bwd_filter(d, dy, x, dw, workspace, workspace_bytes, hip_stream);
}

dl_status dl_bias_relu_bwd_workspace_bytes(int64_t n_pixels, int32_t K, size_t *bytes)
{
    if (!bytes) return DL_ERR_NULL;
    if (n_pixels < 0 || K < 1 || n_pixels * K >= MAX_ELEMS) return DL_ERR_SHAPE;
    *bytes = (size_t)dlk::tail_bwd_blocks(n_pixels, K) * K * sizeof(float);
    return DL_OK;
}

dl_status bias_relu_bwd(const void *dy, const void *y, int32_t dtype, int64_t n_pixels, int32_t K, int32_t relu,
                        void *dz, float *dbias, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dbias) return DL_ERR_NULL;
    if (n_pixels < 0 || K < 1 || n_pixels * K >= MAX_ELEMS) return DL_ERR_SHAPE;
    if (n_pixels > 0 && (!dy || (relu && (!y || !dz)))) return DL_ERR_NULL;
    if (dtype != DL_F16 && dtype != DL_BF16) return DL_ERR_DTYPE;
    if (!aligned16(dy) || !aligned16(y) || !aligned16(dz) || (reinterpret_cast<uintptr_t>(dbias) & 3u)) return DL_ERR_ALIGN;
    const size_t need = (size_t)dlk::tail_bwd_blocks(n_pixels, K) * K * sizeof(float);
    if (!workspace || workspace_bytes < need) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    dlk::TailBwdArgs a{};
    a.dy = static_cast<const uint16_t *>(dy);
    a.y = static_cast<const uint16_t *>(y);
    a.dz = static_cast<uint16_t *>(dz);
    a.partial = static_cast<float *>(workspace);
    a.dbias = dbias;
    a.npix = n_pixels;
    a.K = K;
    a.relu = relu ? 1 : 0;
    return hip_status(dlk::launch_tail_bwd(a, dtype == DL_BF16, static_cast<hipStream_t>(hip_stream)));
}

dl_status dl_larc_workspace_bytes(int32_t n_tensors, size_t *bytes)
{
    if (!bytes) return DL_ERR_NULL;
    if (n_tensors < 0) return DL_ERR_SHAPE;
    *bytes = (size_t)n_tensors * dlk::LARC_SLICES * 2 * sizeof(float);
    return DL_OK;
}

dl_status larc_sgd_step(const dl_larc_tensor *tensors, int32_t n_tensors, int32_t grad_dtype, float lr, float trust,
                        float weight_decay, float momentum, float eps, int32_t clip, float *rates, void *workspace,
                        size_t workspace_bytes, void *hip_stream)
{
    if (n_tensors < 0) return DL_ERR_SHAPE;
    if (n_tensors == 0) return DL_OK;
    if (!tensors) return DL_ERR_NULL;
    if (grad_dtype != DL_F16 && grad_dtype != DL_BF16 && grad_dtype != DL_F32) return DL_ERR_DTYPE;
    for (int i = 0; i < n_tensors; ++i) {
        if (!tensors[i].w || !tensors[i].g) return DL_ERR_NULL;
        if (tensors[i].count < 1 || tensors[i].count >= MAX_ELEMS) return DL_ERR_SHAPE;
        if ((reinterpret_cast<uintptr_t>(tensors[i].w) & 3u) || (reinterpret_cast<uintptr_t>(tensors[i].v) & 3u) ||
            (reinterpret_cast<uintptr_t>(tensors[i].g) & (grad_dtype == DL_F32 ? 3u : 1u)))
            return DL_ERR_ALIGN;
        if (momentum != 0.f && !tensors[i].v) return DL_ERR_NULL;
    }
    const size_t need = (size_t)n_tensors * dlk::LARC_SLICES * 2 * sizeof(float);
    if (!workspace || workspace_bytes < need) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    for (int first = 0; first < n_tensors; first += dlk::LARC_MAX) {
        dlk::LarcBatch b{};
        b.n = n_tensors - first < dlk::LARC_MAX ? n_tensors - first : dlk::LARC_MAX;
        for (int i = 0; i < b.n; ++i) {
            const dl_larc_tensor &t = tensors[first + i];
            b.t[i] = dlk::LarcTensor{static_cast<float *>(t.w), t.g, momentum != 0.f ? static_cast<float *>(t.v) : nullptr,
                                     t.count};
        }
        b.partial = static_cast<float *>(workspace);
        b.rates = rates;
        b.lr = lr; b.trust = trust; b.wd = weight_decay; b.momentum = momentum; b.eps = eps;
        b.clip = clip ? 1 : 0;
        b.first = first;
        if (dlk::launch_larc(b, grad_dtype, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return DL_ERR_LAUNCH;
    }
    return DL_OK;
}

dl_status dl_ce_workspace_bytes(int64_t n_pixels, size_t *bytes)
{
    if (!bytes) return DL_ERR_NULL;
    if (n_pixels < 0) return DL_ERR_SHAPE;
    *bytes = (size_t)dlk::ce_num_blocks(n_pixels) * sizeof(float);
    return DL_OK;
}

namespace {
dl_status run_ce(const void *logits, int32_t dtype, const uint8_t *labels, const float *weights, bool per_pixel,
                 float scale, int64_t n_pixels, float *loss, void *dlogits, void *workspace, size_t workspace_bytes,
                 void *hip_stream)
{
    if (!loss || (!weights && (!per_pixel || n_pixels > 0))) return DL_ERR_NULL;
    if (n_pixels < 0 || n_pixels >= MAX_ELEMS * 16) return DL_ERR_SHAPE;
    if (n_pixels > 0 && (!logits || !labels || !dlogits)) return DL_ERR_NULL;
    if (dtype != DL_F16 && dtype != DL_BF16) return DL_ERR_DTYPE;
    if (!aligned16(logits) || !aligned16(labels) || !aligned16(dlogits) || (per_pixel && !aligned16(weights)))
        return DL_ERR_ALIGN;
    const size_t need = (size_t)dlk::ce_num_blocks(n_pixels) * sizeof(float);
    if (!workspace || workspace_bytes < need) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    return hip_status(dlk::launch_weighted_ce(static_cast<const uint16_t *>(logits), dtype == DL_BF16, labels, weights,
                                              per_pixel, scale, n_pixels, loss, static_cast<uint16_t *>(dlogits),
                                              static_cast<float *>(workspace), static_cast<hipStream_t>(hip_stream)));
}
}  // namespace

dl_status weighted_pixel_ce_fwd_bwd(const void *logits, int32_t dtype, const uint8_t *labels,
                                    const float *class_weights, float scale, int64_t n_pixels, float *loss,
                                    void *dlogits, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_ce(logits, dtype, labels, class_weights, false, scale, n_pixels, loss, dlogits, workspace,
                  workspace_bytes, hip_stream);
}

dl_status weighted_pixel_ce_fwd_bwd_static(const void *logits, int32_t dtype, const uint8_t *labels,
                                           const float *class_weights, float scale, int64_t n_pixels, float *loss,
                                           void *dlogits, void *hip_stream)
{
    // the same checks as the entry point with a workspace, then the size limit of this one
    if (!loss || !class_weights) return DL_ERR_NULL;
    if (n_pixels < 0 || n_pixels > DL_CE_STATIC_MAX_PIXELS) return DL_ERR_SHAPE;
    if (n_pixels > 0 && (!logits || !labels || !dlogits)) return DL_ERR_NULL;
    if (dtype != DL_F16 && dtype != DL_BF16) return DL_ERR_DTYPE;
    if (!aligned16(logits) || !aligned16(labels) || !aligned16(dlogits)) return DL_ERR_ALIGN;
    float *partials = nullptr;
    if (dlk::ce_static_partials(&partials) != hipSuccess) return DL_ERR_LAUNCH;
    return hip_status(dlk::launch_weighted_ce(static_cast<const uint16_t *>(logits), dtype == DL_BF16, labels, class_weights,
                                              false, scale, n_pixels, loss, static_cast<uint16_t *>(dlogits), partials,
                                              static_cast<hipStream_t>(hip_stream)));
}

dl_status weighted_pixel_ce_map_fwd_bwd(const void *logits, int32_t dtype, const uint8_t *labels,
                                        const float *weight_map, float scale, int64_t n_pixels, float *loss,
                                        void *dlogits, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_ce(logits, dtype, labels, weight_map, true, scale, n_pixels, loss, dlogits, workspace, workspace_bytes,
                  hip_stream);
}

}  // extern "C"
