/*
 * fp64 CPU oracle for the convolution + weighted-loss hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU kernels are checked against.  It shares no code with the HIP library,
 * is never linked into it, and must never be called from the product path.
 *
 * What it computes (paper: Sec. "Segmentation Architecture" for convolution
 * and atrous convolution with a dilation factor; Sec. "Weighted loss" for the
 * per-pixel class-weighted loss; Sec. "Performance Measurement" for the
 * (R, S, H, W, C, K, N) naming of a convolution's dimensions):
 *
 *   forward      y[n,p,q,k]  = sum_{r,s,c} x[n, p*st_h - pad_h + r*dil_h,
 *                                             q*st_w - pad_w + s*dil_w, c] * w[k,r,s,c]
 *                (terms whose input coordinate falls outside the image are
 *                 zero: symmetric zero padding; no filter flip)
 *   data grad    dx = (d forward / d x)^T dy, written as the literal transpose
 *                of the forward loop nest (scatter)
 *   filter grad  dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, h(p,r), w(q,s), c]
 *   loss         l_i = -log softmax(z_i)[label_i];  L = scale * sum_i cw[label_i] * l_i
 *                dz_i[c] = scale * cw[label_i] * (softmax(z_i)[c] - [c == label_i])
 *
 * Layouts: activations NHWC, filters KRSC, all dense row-major.  All
 * arithmetic is double precision; every sum runs in the index order written
 * in the loops below (no blocking, no reassociation).
 *
 * The "_at" variants evaluate single output elements from float storage
 * (fp16/bf16 values are exactly representable in float) so that full-size
 * tensors can be spot-checked without holding fp64 copies; the arithmetic is
 * still double.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    int32_t N, H, W, C;           /* input, NHWC */
    int32_t K, R, S;              /* filter, KRSC */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    int32_t dil_h, dil_w;
} oracle_conv_desc;

/* Output extent of one spatial axis: the count of positions p >= 0 such that
 * the last tap, p*st - pad + (R-1)*dil, still lies inside the padded image. */
static int out_extent(int in, int pad, int dil, int taps, int st)
{
    int span = in + 2 * pad - dil * (taps - 1) - 1;
    if (span < 0) return 0;
    return span / st + 1;
}

int oracle_conv_out_shape(const oracle_conv_desc *d, int32_t *P, int32_t *Q)
{
    *P = out_extent(d->H, d->pad_h, d->dil_h, d->R, d->stride_h);
    *Q = out_extent(d->W, d->pad_w, d->dil_w, d->S, d->stride_w);
    return (*P > 0 && *Q > 0) ? 0 : 1;
}

#define XI(n, h, w, c) ((((size_t)(n) * d->H + (h)) * d->W + (w)) * d->C + (c))
#define WI(k, r, s, c) ((((size_t)(k) * d->R + (r)) * d->S + (s)) * d->C + (c))
#define YI(n, p, q, k) ((((size_t)(n) * P + (p)) * Q + (q)) * d->K + (k))

/* ---- forward: the 7-loop definition ------------------------------------ */
void oracle_conv_fwd(const oracle_conv_desc *d, const double *x, const double *w, double *y)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < d->K; ++k) {
                    double acc = 0.0;
                    for (int r = 0; r < d->R; ++r) {
                        int h = p * d->stride_h - d->pad_h + r * d->dil_h;
                        if (h < 0 || h >= d->H) continue;
                        for (int s = 0; s < d->S; ++s) {
                            int ww = q * d->stride_w - d->pad_w + s * d->dil_w;
                            if (ww < 0 || ww >= d->W) continue;
                            for (int c = 0; c < d->C; ++c)
                                acc += x[XI(n, h, ww, c)] * w[WI(k, r, s, c)];
                        }
                    }
                    y[YI(n, p, q, k)] = acc;
                }
}

/* ---- data gradient: transpose of the forward nest (scatter) ------------ */
/* Threads own disjoint channel slices of dx, so no two threads touch the same
 * element and each element's sum runs in (p, q, k, r, s) order. */
void oracle_conv_bwd_data(const oracle_conv_desc *d, const double *dy, const double *w, double *dx)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
    memset(dx, 0, sizeof(double) * (size_t)d->N * d->H * d->W * d->C);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int c = 0; c < d->C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    for (int k = 0; k < d->K; ++k) {
                        double g = dy[YI(n, p, q, k)];
                        for (int r = 0; r < d->R; ++r) {
                            int h = p * d->stride_h - d->pad_h + r * d->dil_h;
                            if (h < 0 || h >= d->H) continue;
                            for (int s = 0; s < d->S; ++s) {
                                int ww = q * d->stride_w - d->pad_w + s * d->dil_w;
                                if (ww < 0 || ww >= d->W) continue;
                                dx[XI(n, h, ww, c)] += g * w[WI(k, r, s, c)];
                            }
                        }
                    }
}

/* ---- filter gradient ---------------------------------------------------- */
/* Each dw element is the sum over (n, p, q) in ascending order.  The channel
 * loop is innermost only so that memory is walked contiguously; it does not
 * change the order in which any single element is accumulated. */
void oracle_conv_bwd_filter(const oracle_conv_desc *d, const double *x, const double *dy, double *dw)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
    memset(dw, 0, sizeof(double) * (size_t)d->K * d->R * d->S * d->C);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < d->K; ++k)
        for (int n = 0; n < d->N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = dy[YI(n, p, q, k)];
                    for (int r = 0; r < d->R; ++r) {
                        int h = p * d->stride_h - d->pad_h + r * d->dil_h;
                        if (h < 0 || h >= d->H) continue;
                        for (int s = 0; s < d->S; ++s) {
                            int ww = q * d->stride_w - d->pad_w + s * d->dil_w;
                            if (ww < 0 || ww >= d->W) continue;
                            for (int c = 0; c < d->C; ++c)
                                dw[WI(k, r, s, c)] += g * x[XI(n, h, ww, c)];
                        }
                    }
                }
}

/* ---- single-element evaluation on float storage ------------------------ */
/* idx holds flat indices into the respective full output tensor. */
void oracle_conv_fwd_at(const oracle_conv_desc *d, const float *x, const float *w,
                        const int64_t *idx, int64_t n_idx, double *out)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int k = (int)(t % d->K); t /= d->K;
        int q = (int)(t % Q);    t /= Q;
        int p = (int)(t % P);    t /= P;
        int n = (int)t;
        double acc = 0.0;
        for (int r = 0; r < d->R; ++r) {
            int h = p * d->stride_h - d->pad_h + r * d->dil_h;
            if (h < 0 || h >= d->H) continue;
            for (int s = 0; s < d->S; ++s) {
                int ww = q * d->stride_w - d->pad_w + s * d->dil_w;
                if (ww < 0 || ww >= d->W) continue;
                for (int c = 0; c < d->C; ++c)
                    acc += (double)x[XI(n, h, ww, c)] * (double)w[WI(k, r, s, c)];
            }
        }
        out[i] = acc;
    }
}

/* dx[n,h,w,c] gathers every (p, r) pair with p*st - pad + r*dil == h (and the
 * same along w): the same set of terms the scatter form adds into it.  For a
 * given tap r the matching p, if any, is (h + pad - r*dil) / st. */
void oracle_conv_bwd_data_at(const oracle_conv_desc *d, const float *dy, const float *w,
                             const int64_t *idx, int64_t n_idx, double *out)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int c  = (int)(t % d->C); t /= d->C;
        int ww = (int)(t % d->W); t /= d->W;
        int h  = (int)(t % d->H); t /= d->H;
        int n  = (int)t;
        double acc = 0.0;
        for (int r = 0; r < d->R; ++r) {
            int th = h + d->pad_h - r * d->dil_h;
            if (th < 0 || th % d->stride_h != 0 || th / d->stride_h >= P) continue;
            int p = th / d->stride_h;
            for (int s = 0; s < d->S; ++s) {
                int tw = ww + d->pad_w - s * d->dil_w;
                if (tw < 0 || tw % d->stride_w != 0 || tw / d->stride_w >= Q) continue;
                int q = tw / d->stride_w;
                for (int k = 0; k < d->K; ++k)
                    acc += (double)dy[YI(n, p, q, k)] * (double)w[WI(k, r, s, c)];
            }
        }
        out[i] = acc;
    }
}

void oracle_conv_bwd_filter_at(const oracle_conv_desc *d, const float *x, const float *dy,
                               const int64_t *idx, int64_t n_idx, double *out)
{
    int32_t P, Q;
    oracle_conv_out_shape(d, &P, &Q);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int c = (int)(t % d->C); t /= d->C;
        int s = (int)(t % d->S); t /= d->S;
        int r = (int)(t % d->R); t /= d->R;
        int k = (int)t;
        double acc = 0.0;
        for (int n = 0; n < d->N; ++n)
            for (int p = 0; p < P; ++p) {
                int h = p * d->stride_h - d->pad_h + r * d->dil_h;
                if (h < 0 || h >= d->H) continue;
                for (int q = 0; q < Q; ++q) {
                    int ww = q * d->stride_w - d->pad_w + s * d->dil_w;
                    if (ww < 0 || ww >= d->W) continue;
                    acc += (double)dy[YI(n, p, q, k)] * (double)x[XI(n, h, ww, c)];
                }
            }
        out[i] = acc;
    }
}

/* ---- class-weighted per-pixel softmax cross-entropy --------------------- */
/* n_classes is a parameter so that textbook special cases can be pinned; the
 * workload uses 3.  The loss is accumulated pixel by pixel in index order. */
void oracle_weighted_ce(const double *z, const uint8_t *labels, const double *cw, double scale,
                        int64_t n_pixels, int32_t n_classes, double *loss, double *dz)
{
    double total = 0.0;
    for (int64_t i = 0; i < n_pixels; ++i) {
        const double *zi = z + (size_t)i * n_classes;
        int lab = labels[i];
        double m = zi[0];
        for (int c = 1; c < n_classes; ++c)
            if (zi[c] > m) m = zi[c];
        double se = 0.0;
        for (int c = 0; c < n_classes; ++c) se += exp(zi[c] - m);
        double lse = m + log(se);
        double wi = cw[lab];
        total += wi * (lse - zi[lab]);
        if (dz) {
            for (int c = 0; c < n_classes; ++c) {
                double pc = exp(zi[c] - lse);
                dz[(size_t)i * n_classes + c] = scale * wi * (pc - (c == lab ? 1.0 : 0.0));
            }
        }
    }
    *loss = scale * total;
}

/* ---- the same loss with the weight given per pixel ------------------------ */
/* Sec. "Weighted loss": the per-pixel weight map is computed by the input
 * pipeline and handed to the GPU with the image.  l_i and the softmax are as
 * above; the weight of pixel i is wmap[i] instead of cw[label_i]. */
void oracle_weighted_ce_map(const double *z, const uint8_t *labels, const double *wmap, double scale,
                            int64_t n_pixels, int32_t n_classes, double *loss, double *dz)
{
    double total = 0.0;
    for (int64_t i = 0; i < n_pixels; ++i) {
        const double *zi = z + (size_t)i * n_classes;
        int lab = labels[i];
        double m = zi[0];
        for (int c = 1; c < n_classes; ++c)
            if (zi[c] > m) m = zi[c];
        double se = 0.0;
        for (int c = 0; c < n_classes; ++c) se += exp(zi[c] - m);
        double lse = m + log(se);
        total += wmap[i] * (lse - zi[lab]);
        if (dz) {
            for (int c = 0; c < n_classes; ++c) {
                double pc = exp(zi[c] - lse);
                dz[(size_t)i * n_classes + c] = scale * wmap[i] * (pc - (c == lab ? 1.0 : 0.0));
            }
        }
    }
    *loss = scale * total;
}
