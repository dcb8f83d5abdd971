/*
 * Sanitizer run of the library's HOST code (argument validation, workspace sizing, kernel and tile
 * planning): built by tests/test_sanitizers.py against a copy of the library whose host side is
 * compiled with -fsanitize=address,undefined.  No GPU is touched: every call here either fails
 * validation before any launch or is a planning query (dl_conv_describe walks the entry points'
 * dispatch with launches turned into log lines).
 */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../include/dlconv.h"

static int sweep(void)
{
    static const int Hs[] = {1, 3, 17, 48, 150, 768}, Ws[] = {1, 5, 33, 72, 170, 1152};
    static const int Cs[] = {1, 3, 8, 16, 40, 64, 256, 304, 1024, 2048}, Ks[] = {1, 3, 8, 32, 48, 64, 160, 256, 304, 2048};
    static const int Rs[] = {1, 3, 5, 7}, Ss[] = {1, 2, 3}, Ds[] = {1, 2, 6, 18};
    int n = 0;
    char buf[512];
    for (unsigned hi = 0; hi < 6; ++hi)
        for (unsigned ci = 0; ci < 10; ++ci)
            for (unsigned ki = 0; ki < 10; ++ki)
                for (unsigned ri = 0; ri < 4; ++ri)
                    for (unsigned si = 0; si < 3; ++si)
                        for (unsigned di = 0; di < 4; ++di) {
                            if ((hi + ci + ki + ri + si + di) % 3 != 0) continue;          /* a third of the grid */
                            dl_conv_desc d = {2, Hs[hi], Ws[hi], Cs[ci], Ks[ki], Rs[ri], Rs[ri], Ss[si], Ss[si],
                                              Ds[di] * (Rs[ri] / 2), Ds[di] * (Rs[ri] / 2), Ds[di], Ds[di], (int32_t)((ci + ki) & 1), 0};
                            d.dw_dtype = (di & 1) ? DL_F32 : d.dtype;
                            int32_t P, Q;
                            if (dl_conv_out_shape(&d, &P, &Q) != DL_OK) continue;
                            for (int pass = 0; pass < 3; ++pass) {
                                size_t bytes = 0;
                                if (dl_conv_workspace_bytes(&d, pass, &bytes) != DL_OK) return -1;
                                if (dl_conv_describe(&d, pass, buf, sizeof buf) != DL_OK) return -2;
                                if (strlen(buf) == 0) return -3;
                            }
                            ++n;
                        }
    return n;
}

int main(void)
{
    const int n = sweep();
    if (n < 500) { printf("sweep failed: %d\n", n); return 1; }
    dl_conv_desc d = {1, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, DL_F16, DL_F16};
    void *p16 = (void *)16, *p24 = (void *)24;
    int bad = 0;
    bad += conv2d_fwd(&d, NULL, NULL, NULL, NULL, 0, NULL) != DL_ERR_NULL;
    bad += conv2d_fwd(&d, p16, p16, p24, NULL, 0, NULL) != DL_ERR_ALIGN;
    bad += conv2d_bwd_data(&d, p16, p16, p16, NULL, 0, NULL) != DL_ERR_WORKSPACE;
    bad += conv2d_bwd_filter(&d, p16, p16, p16, (void *)32, 8, NULL) != DL_ERR_WORKSPACE;
    bad += conv2d_transpose_fwd(&d, p16, p16, p24, NULL, 0, NULL) != DL_ERR_ALIGN;
    bad += conv2d_fwd_bias_relu(&d, p16, p16, (const float *)18, 1, p16, NULL, 0, NULL) != DL_ERR_ALIGN;
    bad += weighted_pixel_ce_fwd_bwd(p16, 0, p16, p16, 1.0f, -1, p16, p16, p16, 64, NULL) != DL_ERR_SHAPE;
    bad += weighted_pixel_ce_fwd_bwd_static(p16, 0, p16, p16, 1.0f, DL_CE_STATIC_MAX_PIXELS + 1, p16, p16, NULL) != DL_ERR_SHAPE;
    bad += weighted_pixel_ce_map_fwd_bwd(p16, 0, p16, NULL, 1.0f, 8, p16, p16, p16, 64, NULL) != DL_ERR_NULL;
    bad += logits_ce_fused_fwd_bwd(p16, p16, 0, p16, p16, 1.0f, 8, 24, p16, p16, p16, p16, p16, 0, p16, 1 << 20, NULL) != DL_ERR_SHAPE;
    bad += bias_relu_bwd(p16, p16, 0, 8, 0, 1, p16, p16, p16, 4096, NULL) != DL_ERR_SHAPE;
    dl_larc_tensor t[2] = {{p16, p16, NULL, 8}, {p16, NULL, NULL, 8}};
    bad += larc_sgd_step(t, 2, 0, .1f, .02f, 0.f, 0.f, 0.f, 1, NULL, p16, 1 << 20, NULL) != DL_ERR_NULL;
    size_t bytes;
    bad += dl_ce_workspace_bytes(2 * 768 * 1152, &bytes) != DL_OK;
    bad += dl_logits_ce_workspace_bytes(2 * 768 * 1152, 256, &bytes) != DL_OK;
    bad += dl_bias_relu_bwd_workspace_bytes(2 * 768 * 1152, 256, &bytes) != DL_OK;
    bad += dl_larc_workspace_bytes(63, &bytes) != DL_OK;
    printf("host-path sanitizer run: %d descriptors planned, %d wrong status codes\n", n, bad);
    return bad != 0;
}
