// C boundary: argument validation, workspace sizing, and the mapping of the
// three convolution passes and the loss onto the gfx950 kernels.  Everything
// here runs on the host; validation happens before any launch.
#include <hip/hip_runtime.h>

#include "../../include/dlconv.h"
#include "kernels.h"

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

size_t dgrad_workspace(const dl_conv_desc *d)
{
    // one re-laid-out filter slice per stride-parity class, each 256-byte aligned
    size_t total = 0;
    for (int a = 0; a < d->stride_h; ++a)
        for (int b = 0; b < d->stride_w; ++b) {
            const AxisTaps th = class_taps(a, d->R, d->stride_h, d->pad_h, d->dil_h);
            const AxisTaps tw = class_taps(b, d->S, d->stride_w, d->pad_w, d->dil_w);
            total += align_up((size_t)d->C * th.count * tw.count * d->K * sizeof(uint16_t), 256);
        }
    return total;
}

dlk::WgradPlan wgrad_plan(const dl_conv_desc *d, const Geometry &g)
{
    return dlk::wgrad_make_plan((int64_t)d->N * g.P * g.Q, d->K, d->C, d->R * d->S * d->C);
}

size_t wgrad_workspace(const dl_conv_desc *d, const Geometry &g)
{
    return (size_t)wgrad_plan(d, g).splits * (size_t)g.w_elems * sizeof(float);
}

dl_status hip_status(hipError_t e) { return e == hipSuccess ? DL_OK : DL_ERR_LAUNCH; }

}  // namespace

extern "C" {

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
        case DL_PASS_FWD: *bytes = 0; return DL_OK;
        case DL_PASS_BWD_DATA: *bytes = dgrad_workspace(desc); return DL_OK;
        case DL_PASS_BWD_FILTER: *bytes = wgrad_workspace(desc, g); return DL_OK;
    }
    return DL_ERR_UNSUPPORTED;
}

dl_status conv2d_fwd(const dl_conv_desc *d, const void *x, const void *w, void *y, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (!d || !x || !w || !y) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return DL_ERR_ALIGN;

    dlk::IgemmArgs a{};
    a.A = static_cast<const uint16_t *>(x);
    a.B = static_cast<const uint16_t *>(w);
    a.D = static_cast<uint16_t *>(y);
    a.NB = d->N; a.IH = d->H; a.IW = d->W; a.Cin = d->C;
    a.OH = g.P; a.OW = g.Q; a.Nout = d->K;
    a.TR = d->R; a.TS = d->S;
    a.sh = d->stride_h; a.sw = d->stride_w;
    a.th0 = -d->pad_h; a.dth = d->dil_h; a.tw0 = -d->pad_w; a.dtw = d->dil_w;
    a.FH = g.P; a.FW = g.Q; a.osh = 1; a.osw = 1; a.ooh = 0; a.oow = 0; a.ldd = d->K;
    return hip_status(dlk::launch_igemm(a, d->dtype == DL_BF16, static_cast<hipStream_t>(hip_stream)));
}

dl_status conv2d_bwd_data(const dl_conv_desc *d, const void *dy, const void *w, void *dx, void *workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    if (!d || !dy || !w || !dx) return DL_ERR_NULL;
    Geometry g;
    const dl_status st = check_desc(d, &g);
    if (st != DL_OK) return st;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return DL_ERR_ALIGN;
    const size_t need = dgrad_workspace(d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return DL_ERR_WORKSPACE;
    if (need > 0 && !aligned16(workspace)) return DL_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // Input pixels (h, w) fall into stride_h*stride_w parity classes; within a
    // class the contributing taps and the output pixels they pair with form
    // regular grids, so each class is one dense implicit GEMM over dy.
    size_t ws_off = 0;
    for (int ca = 0; ca < d->stride_h; ++ca)
        for (int cb = 0; cb < d->stride_w; ++cb) {
            const int OH = ca < d->H ? (d->H - ca + d->stride_h - 1) / d->stride_h : 0;
            const int OW = cb < d->W ? (d->W - cb + d->stride_w - 1) / d->stride_w : 0;
            const AxisTaps th = class_taps(ca, d->R, d->stride_h, d->pad_h, d->dil_h);
            const AxisTaps tw = class_taps(cb, d->S, d->stride_w, d->pad_w, d->dil_w);
            const size_t slice = align_up((size_t)d->C * th.count * tw.count * d->K * sizeof(uint16_t), 256);
            uint16_t *wt = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) + ws_off);
            ws_off += slice;
            if (OH == 0 || OW == 0) continue;
            const bool has_taps = th.count > 0 && tw.count > 0;
            if (has_taps) {
                dlk::FilterRelayoutArgs f{};
                f.w = static_cast<const uint16_t *>(w);
                f.wt = wt;
                f.K = d->K; f.R = d->R; f.S = d->S; f.C = d->C;
                f.r0 = th.r0; f.rstep = th.rstep; f.TR = th.count;
                f.s0 = tw.r0; f.sstep = tw.rstep; f.TS = tw.count;
                const hipError_t e = dlk::launch_filter_relayout(f, stream);
                if (e != hipSuccess) return DL_ERR_LAUNCH;
            }
            dlk::IgemmArgs a{};
            a.A = static_cast<const uint16_t *>(dy);
            a.B = has_taps ? wt : static_cast<const uint16_t *>(w);   // never read when there are no taps
            a.D = static_cast<uint16_t *>(dx);
            a.NB = d->N; a.IH = g.P; a.IW = g.Q; a.Cin = d->K;
            a.OH = OH; a.OW = OW; a.Nout = d->C;
            a.TR = has_taps ? th.count : 0; a.TS = has_taps ? tw.count : 1;
            a.sh = 1; a.sw = 1;
            a.th0 = th.t0; a.dth = th.dt; a.tw0 = tw.t0; a.dtw = tw.dt;
            a.FH = d->H; a.FW = d->W; a.osh = d->stride_h; a.osw = d->stride_w; a.ooh = ca; a.oow = cb;
            a.ldd = d->C;
            const hipError_t e = dlk::launch_igemm(a, d->dtype == DL_BF16, stream);
            if (e != hipSuccess) return DL_ERR_LAUNCH;
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
    hipError_t e = plan.cfg >= 0 ? dlk::launch_wgrad_dma(a, d->dtype == DL_BF16, plan.cfg, stream)
                                 : dlk::launch_wgrad(a, d->dtype == DL_BF16, stream);
    if (e != hipSuccess) return DL_ERR_LAUNCH;
    e = dlk::launch_splitk_reduce(a.partial, plan.splits, g.w_elems, dw, d->dw_dtype, stream);
    return hip_status(e);
}

dl_status dl_ce_workspace_bytes(int64_t n_pixels, size_t *bytes)
{
    if (!bytes) return DL_ERR_NULL;
    if (n_pixels < 0) return DL_ERR_SHAPE;
    *bytes = (size_t)dlk::ce_num_blocks(n_pixels) * sizeof(float);
    return DL_OK;
}

dl_status weighted_pixel_ce_fwd_bwd(const void *logits, int32_t dtype, const uint8_t *labels,
                                    const float *class_weights, float scale, int64_t n_pixels, float *loss,
                                    void *dlogits, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!class_weights || !loss) return DL_ERR_NULL;
    if (n_pixels < 0 || n_pixels >= MAX_ELEMS * 16) return DL_ERR_SHAPE;
    if (n_pixels > 0 && (!logits || !labels || !dlogits)) return DL_ERR_NULL;
    if (dtype != DL_F16 && dtype != DL_BF16) return DL_ERR_DTYPE;
    if (!aligned16(logits) || !aligned16(labels) || !aligned16(dlogits)) return DL_ERR_ALIGN;
    const size_t need = (size_t)dlk::ce_num_blocks(n_pixels) * sizeof(float);
    if (!workspace || workspace_bytes < need) return DL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DL_ERR_ALIGN;
    return hip_status(dlk::launch_weighted_ce(static_cast<const uint16_t *>(logits), dtype == DL_BF16, labels,
                                              class_weights, scale, n_pixels, loss,
                                              static_cast<uint16_t *>(dlogits), static_cast<float *>(workspace),
                                              static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
