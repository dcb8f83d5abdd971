// The logits layer fused with the loss (gfx950): the 1x1 convolution from C
// channels to the 3 classes, the class-weighted softmax cross-entropy and both
// gradients of that convolution in ONE pass over the C-channel activation
// tensor.  As four separate calls (forward, loss, data gradient, filter
// gradient) the tensor is read twice and its gradient written once, with the
// 3-channel logits and their gradient travelling through memory in between;
// here it is read once and its gradient written once: 4*C + 1 bytes per pixel.
//
//   z_i = W x_i;  loss = scale * sum_i cw[label_i] * (logsumexp(z_i) - z_i[label_i])
//   dz_i = scale * cw[label_i] * (softmax(z_i) - onehot(label_i));  dx_i = W^T dz_i;  dW = sum_i dz_i x_i^T
//
// A thread owns one 16-byte chunk (8 channels) of a pixel; the G = C/8 threads
// of a pixel leave their partial dot products in LDS, one thread per pixel adds
// them in chunk order, evaluates the loss in fp32 (nothing is rounded between the
// steps; the optional logits / dlogits copies are rounded on store) and hands
// dz back through LDS; every thread then forms its chunk of dx from the activation
// chunk it still holds and adds dz x^T to 24 running sums of dW.  A workgroup
// handles 4 * (256 / G) pixels per trip (two barriers), with the next trip's
// loads already issued.  Workgroup sums of dW and of the loss are added by
// pixel slot in a fixed order and written as partials; an ordered reduce
// follows: no atomics, run-to-run identical.
#include "device_common.h"
#include "kernels.h"

namespace dlk {

namespace {
constexpr int LC_THREADS = 256, LC_U = 4, LC_MAX_BLOCKS = 2048;
}

template <class T>
__global__ __launch_bounds__(LC_THREADS) void logits_ce_kernel(const LogitsCeArgs p)
{
    const int G = p.C / 8;                               // threads (chunks) per pixel, <= 256
    const int PPI = LC_THREADS / G;                      // pixels per pass
    const int PB = LC_U * PPI;                           // pixels per trip
    // one buffer: during the trips the partial dot products [pixel slot q][class][chunk] (12 KB at most),
    // at the end the 24 running sums of every thread
    __shared__ float buf[LC_THREADS * 24];
    __shared__ float dzs[LC_THREADS][4];                 // [pixel slot q]: dz (PB <= 256: C >= 32)
    float *const pd = buf, *const red = buf;

    const int tid = threadIdx.x, g = tid % G, ps = tid / G;
    const bool active = ps < PPI;
    float wv[3][8];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const u32x4_t v = active ? *reinterpret_cast<const u32x4_t *>(p.w + (size_t)k * p.C + g * 8) : u32x4_t{0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            wv[k][2 * d] = T::to_float((uint16_t)(v[d] & 0xffffu));
            wv[k][2 * d + 1] = T::to_float((uint16_t)(v[d] >> 16));
        }
    }
    const float cw0 = p.cw[0], cw1 = p.cw[1], cw2 = p.cw[2];
    float acc[3][8];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    float loss_sum = 0.f;

    const int64_t ntrips = (p.n + PB - 1) / PB;
    u32x4_t nx[LC_U];
    auto fetch = [&](int64_t trip) {
#pragma unroll
        for (int u = 0; u < LC_U; ++u) {
            const int64_t pix = trip * PB + u * PPI + ps;
            nx[u] = (active && pix < p.n) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p.x + pix * p.C + g * 8))
                                          : u32x4_t{0, 0, 0, 0};
        }
    };
    if ((int64_t)blockIdx.x < ntrips) fetch(blockIdx.x);
    for (int64_t trip = blockIdx.x; trip < ntrips; trip += gridDim.x) {
        float xf[LC_U][8];
#pragma unroll
        for (int u = 0; u < LC_U; ++u)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                xf[u][2 * d] = T::to_float((uint16_t)(nx[u][d] & 0xffffu));
                xf[u][2 * d + 1] = T::to_float((uint16_t)(nx[u][d] >> 16));
            }
        if (trip + gridDim.x < ntrips) fetch(trip + gridDim.x);
        // ---- partial dot products of this chunk ------------------------------------
        if (active) {
#pragma unroll
            for (int u = 0; u < LC_U; ++u) {
                const int q = u * PPI + ps;
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    float s = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) s += xf[u][e] * wv[k][e];
                    pd[(q * 3 + k) * G + g] = s;
                }
            }
        }
        __syncthreads();
        // ---- one thread per pixel: logits, loss, dz -----------------------------------
        if (tid < PB) {
            const int q = tid;
            const int64_t pix = trip * PB + q;
            float z[3] = {0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const float *src = pd + (q * 3 + k) * G;
                float s = 0.f;
                for (int c = 0; c < G; ++c) s += src[c];                 // chunk order: fixed
                z[k] = s;
            }
            float d0 = 0.f, d1 = 0.f, d2 = 0.f;
            if (pix < p.n) {
                if (p.logits) {
                    p.logits[pix * 3] = T::from_float(z[0]);
                    p.logits[pix * 3 + 1] = T::from_float(z[1]);
                    p.logits[pix * 3 + 2] = T::from_float(z[2]);
                }
                const int lab = p.labels[pix];
                const float wl = lab == 0 ? cw0 : (lab == 1 ? cw1 : cw2);
                const float m = fmaxf(z[0], fmaxf(z[1], z[2]));
                const float e0 = __expf(z[0] - m), e1 = __expf(z[1] - m), e2 = __expf(z[2] - m);
                const float se = e0 + e1 + e2;
                const float zl = lab == 0 ? z[0] : (lab == 1 ? z[1] : z[2]);
                loss_sum += wl * (m + __logf(se) - zl);
                const float gsc = p.scale * wl / se;
                d0 = gsc * e0 - (lab == 0 ? p.scale * wl : 0.f);
                d1 = gsc * e1 - (lab == 1 ? p.scale * wl : 0.f);
                d2 = gsc * e2 - (lab == 2 ? p.scale * wl : 0.f);
                if (p.dlogits) {
                    p.dlogits[pix * 3] = T::from_float(d0);
                    p.dlogits[pix * 3 + 1] = T::from_float(d1);
                    p.dlogits[pix * 3 + 2] = T::from_float(d2);
                }
            }
            dzs[q][0] = d0; dzs[q][1] = d1; dzs[q][2] = d2;
        }
        __syncthreads();
        // ---- this chunk of dx, and dz x^T into the running sums of dW ---------------------
        if (active) {
#pragma unroll
            for (int u = 0; u < LC_U; ++u) {
                const int q = u * PPI + ps;
                const int64_t pix = trip * PB + q;
                const float d0 = dzs[q][0], d1 = dzs[q][1], d2 = dzs[q][2];
                u32x4_t out;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const float a = d0 * wv[0][2 * d] + d1 * wv[1][2 * d] + d2 * wv[2][2 * d];
                    const float b = d0 * wv[0][2 * d + 1] + d1 * wv[1][2 * d + 1] + d2 * wv[2][2 * d + 1];
                    out[d] = (uint32_t)T::from_float(a) | ((uint32_t)T::from_float(b) << 16);
                }
                if (pix < p.n) __builtin_nontemporal_store(out, reinterpret_cast<u32x4_t *>(p.dx + pix * p.C + g * 8));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    acc[0][e] += d0 * xf[u][e];
                    acc[1][e] += d1 * xf[u][e];
                    acc[2][e] += d2 * xf[u][e];
                }
            }
        }
        // (the next trip writes pd only after this barrier-separated phase: every thread is past its
        //  reads of pd; it reads dzs only after its own first barrier, by which time every thread has
        //  finished this phase)
    }
    // ---- workgroup sums: dW by pixel slot in order, the loss by thread in order --------------
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) red[(k * 8 + e) * LC_THREADS + tid] = active ? acc[k][e] : 0.f;
    __syncthreads();
    float *out_dw = p.partial_dw + (size_t)blockIdx.x * 3 * p.C;
    for (int i = tid; i < 3 * p.C; i += LC_THREADS) {
        const int k = i / p.C, c = i - k * p.C;
        const int gg = c >> 3, e = c & 7;
        const float *src = red + (k * 8 + e) * LC_THREADS + gg;
        float s = 0.f;
        for (int slot = 0; slot < PPI; ++slot) s += src[slot * G];
        out_dw[i] = s;
    }
    __syncthreads();
    red[tid] = loss_sum;
    __syncthreads();
    if (tid == 0) {
        float s = 0.f;
        for (int i = 0; i < LC_THREADS; ++i) s += red[i];
        p.partial_loss[blockIdx.x] = s;
    }
}

int logits_ce_blocks(int64_t n_pixels, int C)
{
    const int G = C / 8, PB = LC_U * (LC_THREADS / (G > 0 ? G : 1));
    int64_t b = (n_pixels + PB - 1) / PB;
    if (b > LC_MAX_BLOCKS) b = LC_MAX_BLOCKS;
    if (b < 1) b = 1;
    return (int)b;
}

hipError_t launch_logits_ce(const LogitsCeArgs &a, bool is_bf16, hipStream_t stream)
{
    if (a.C % 8 != 0 || a.C < 32 || a.C > 2048 || a.n < 0) return hipErrorInvalidValue;   // 4..256 chunks per pixel
    const dim3 grid(logits_ce_blocks(a.n, a.C)), block(LC_THREADS);
    if (is_bf16) hipLaunchKernelGGL(logits_ce_kernel<BF16>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(logits_ce_kernel<F16>, grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace dlk
