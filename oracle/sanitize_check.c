/*
 * Sanitizer run of the fp64 oracle (TEST INFRASTRUCTURE, like oracle.c itself): built by
 * tests/test_sanitizers.py together with oracle.c under -fsanitize=address,undefined and run on
 * small geometries that reach every branch of the index arithmetic (padding on all sides, taps
 * that fall entirely into the padding, strides that skip the last rows, dilation, 1x1, single
 * pixel).  It checks nothing numerically (the pins in tests/ do that); it exists so that an
 * out-of-bounds index or an overflow in the oracle cannot hide behind a plausible number.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int32_t N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_conv_desc;

int oracle_conv_out_shape(const oracle_conv_desc *d, int32_t *P, int32_t *Q);
void oracle_conv_fwd(const oracle_conv_desc *d, const double *x, const double *w, double *y);
void oracle_conv_bwd_data(const oracle_conv_desc *d, const double *dy, const double *w, double *dx);
void oracle_conv_bwd_filter(const oracle_conv_desc *d, const double *x, const double *dy, double *dw);
void oracle_conv_fwd_at(const oracle_conv_desc *d, const float *x, const float *w, const int64_t *idx, int64_t n, double *out);
void oracle_conv_bwd_data_at(const oracle_conv_desc *d, const float *dy, const float *w, const int64_t *idx, int64_t n, double *out);
void oracle_conv_bwd_filter_at(const oracle_conv_desc *d, const float *x, const float *dy, const int64_t *idx, int64_t n, double *out);
void oracle_weighted_ce(const double *z, const uint8_t *labels, const double *cw, double scale, int64_t n, int32_t nc, double *loss, double *dz);
void oracle_weighted_ce_map(const double *z, const uint8_t *labels, const double *wm, double scale, int64_t n, int32_t nc, double *loss, double *dz);

static double *dbuf(size_t n) { double *p = malloc(sizeof(double) * (n ? n : 1)); for (size_t i = 0; i < n; ++i) p[i] = (double)((i * 2654435761u) % 17) - 8.0; return p; }
static float *fbuf(size_t n) { float *p = malloc(sizeof(float) * (n ? n : 1)); for (size_t i = 0; i < n; ++i) p[i] = (float)((i * 40503u) % 13) - 6.0f; return p; }

int main(void)
{
    static const oracle_conv_desc cases[] = {
        {1, 5, 6, 2, 3, 3, 3, 1, 1, 1, 1, 1, 1}, {2, 7, 5, 3, 4, 3, 3, 2, 2, 1, 1, 1, 1}, {1, 9, 9, 2, 2, 3, 3, 1, 1, 6, 6, 6, 6},
        {1, 4, 4, 1, 1, 3, 3, 1, 1, 18, 18, 18, 18}, {1, 11, 13, 2, 3, 7, 7, 2, 2, 3, 3, 1, 1}, {2, 6, 7, 5, 3, 1, 1, 1, 1, 0, 0, 1, 1},
        {1, 6, 7, 4, 2, 1, 1, 2, 2, 0, 0, 1, 1}, {1, 3, 3, 2, 2, 3, 3, 1, 1, 0, 0, 1, 1}, {1, 8, 9, 2, 2, 3, 1, 2, 3, 1, 0, 2, 1},
        {1, 10, 8, 1, 2, 5, 5, 3, 3, 2, 2, 1, 1}, {1, 1, 1, 8, 4, 1, 1, 1, 1, 0, 0, 1, 1}, {1, 7, 7, 2, 2, 3, 3, 3, 3, 2, 2, 2, 2}};
    int runs = 0;
    for (size_t c = 0; c < sizeof cases / sizeof cases[0]; ++c) {
        const oracle_conv_desc *d = &cases[c];
        int32_t P, Q;
        if (oracle_conv_out_shape(d, &P, &Q)) continue;
        const size_t nx = (size_t)d->N * d->H * d->W * d->C, nw = (size_t)d->K * d->R * d->S * d->C, ny = (size_t)d->N * P * Q * d->K;
        double *x = dbuf(nx), *w = dbuf(nw), *y = dbuf(ny), *dx = dbuf(nx), *dw = dbuf(nw);
        oracle_conv_fwd(d, x, w, y);
        oracle_conv_bwd_data(d, y, w, dx);
        oracle_conv_bwd_filter(d, x, y, dw);
        float *xf = fbuf(nx), *wf = fbuf(nw), *yf = fbuf(ny);
        int64_t *ix = malloc(sizeof(int64_t) * (nx + nw + ny));
        double *out = malloc(sizeof(double) * (nx + nw + ny));
        for (size_t i = 0; i < ny; ++i) ix[i] = (int64_t)i;
        oracle_conv_fwd_at(d, xf, wf, ix, (int64_t)ny, out);
        for (size_t i = 0; i < nx; ++i) ix[i] = (int64_t)i;
        oracle_conv_bwd_data_at(d, yf, wf, ix, (int64_t)nx, out);
        for (size_t i = 0; i < nw; ++i) ix[i] = (int64_t)i;
        oracle_conv_bwd_filter_at(d, xf, yf, ix, (int64_t)nw, out);
        free(x); free(w); free(y); free(dx); free(dw); free(xf); free(wf); free(yf); free(ix); free(out);
        ++runs;
    }
    for (int n = 0; n < 40; n += 13) {
        double *z = dbuf((size_t)n * 3), *dz = dbuf((size_t)n * 3), *wm = dbuf((size_t)n);
        uint8_t *lab = malloc(n ? n : 1);
        for (int i = 0; i < n; ++i) lab[i] = (uint8_t)(i % 3);
        const double cw[3] = {1.0, 7.7, 31.6};
        double loss;
        oracle_weighted_ce(z, lab, cw, 0.5, n, 3, &loss, dz);
        oracle_weighted_ce(z, lab, cw, 0.5, n, 3, &loss, NULL);
        oracle_weighted_ce_map(z, lab, wm, 0.5, n, 3, &loss, dz);
        free(z); free(dz); free(wm); free(lab);
    }
    printf("oracle sanitizer run: %d geometries ok\n", runs);
    return runs >= 10 ? 0 : 1;
}
