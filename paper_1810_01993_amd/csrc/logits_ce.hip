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
// A thread owns one 16-byte chunk (8 channels) of a pixel.  The G = C/8 threads
// of a pixel add their partial dot products; the loss is evaluated in fp32
// (nothing is rounded between the steps; the optional logits / dlogits copies
// are rounded on store); every thread then forms its chunk of dx from the
// activation chunk it still holds and adds dz x^T to 24 running sums of dW.
// When G is 32 (C = 256: the network's layer) a pixel is half a wavefront: four
// DPP row shifts add each row of 16 lanes, four lane reads and two scalar adds
// give the two pixels' sums, every lane evaluates the (cheap) loss itself, and
// the trips need no LDS and no barrier.  Otherwise the partial sums go
// through LDS, one thread per pixel adds them in chunk order and hands dz back
// (two barriers per trip).  A workgroup handles 2 * (256 / G) pixels per trip,
// with the next trip's loads already issued.  Workgroup sums of dW and of the
// loss are added by pixel slot in a fixed order and written as partials; an
// ordered reduce follows: no atomics, run-to-run identical.
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace dlk {

namespace {
constexpr int LC_THREADS = 256, LC_U = 2, LC_MAX_BLOCKS = 2048;

// v summed over lanes 0..31 (returned in lanes 0..31) and over lanes 32..63 (in lanes 32..63), in a fixed order.
__device__ __forceinline__ float half_wave_sum(float v, int lane)
{
    auto shr = [](float t, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    float t = v;                                         // row_shr:n reads lane - n of the same row of 16, zero outside it
    t += shr(t, std::integral_constant<int, 0x111>{});
    t += shr(t, std::integral_constant<int, 0x112>{});
    t += shr(t, std::integral_constant<int, 0x114>{});
    t += shr(t, std::integral_constant<int, 0x118>{});   // lane 15 of every row: the row's sum
    auto at = [&](int l) { return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t), l)); };
    const float lo = at(15) + at(31);
    const float hi = at(47) + at(63);
    return lane < 32 ? lo : hi;
}
}

template <class T, bool SHFL>
__global__ __launch_bounds__(LC_THREADS, 3) void logits_ce_kernel(const LogitsCeArgs args)
{
    // (the fields as plain locals: captured by reference inside the lambdas below, the argument struct itself
    // would be given a home in scratch memory)
    const uint16_t *const a_x = args.x, *const a_w = args.w;
    const uint8_t *const a_labels = args.labels;
    const float *const a_cw = args.cw;
    const float a_scale = args.scale;
    const int64_t a_n = args.n;
    const int a_C = args.C;
    uint16_t *const a_logits = args.logits, *const a_dlogits = args.dlogits, *const a_dx = args.dx;
    float *const a_partial_dw = args.partial_dw, *const a_partial_loss = args.partial_loss;
    const int G = a_C / 8;                               // threads (chunks) per pixel, <= 256
    const int PPI = LC_THREADS / G;                      // pixels per pass
    const int PB = LC_U * PPI;                           // pixels per trip
    // one buffer: during the trips the partial dot products [pixel slot q][class][chunk] (6 KB at most),
    // at the end the 24 running sums of every thread
    __shared__ float buf[LC_THREADS * 24];
    __shared__ float dzs[LC_THREADS][4];                 // [pixel slot q]: dz (PB <= 256: C >= 32)
    float *const pd = buf, *const red = buf;

    const int tid = threadIdx.x, g = tid % G, ps = tid / G;
    const bool active = ps < PPI;
    float wv[3][8];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const u32x4_t v = active ? *reinterpret_cast<const u32x4_t *>(a_w + (size_t)k * a_C + g * 8) : u32x4_t{0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            wv[k][2 * d] = T::to_float((uint16_t)(v[d] & 0xffffu));
            wv[k][2 * d + 1] = T::to_float((uint16_t)(v[d] >> 16));
        }
    }
    const float cw0 = a_cw[0], cw1 = a_cw[1], cw2 = a_cw[2];
    float acc[3][8];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    float loss_sum = 0.f;

    const int64_t ntrips = (a_n + PB - 1) / PB;
    u32x4_t nx[LC_U];
    int nlab[LC_U];                                      // SHFL: the labels of this thread's pixels
    int nlab1 = 0;                                       // otherwise: the label of pixel slot tid
    auto fetch = [&](int64_t trip) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < LC_U; ++u) {
            const int64_t pix = trip * PB + u * PPI + ps;
            nx[u] = (active && pix < a_n) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(a_x + pix * a_C + g * 8))
                                          : u32x4_t{0, 0, 0, 0};
            if (SHFL) nlab[u] = pix < a_n ? a_labels[pix] : 0;
        }
        // fetched with the activations, a trip ahead: a load issued later would be waited for in order,
        // i.e. together with everything fetched ahead
        if (!SHFL) nlab1 = (tid < PB && trip * PB + tid < a_n) ? a_labels[trip * PB + tid] : 0;
    };
    if ((int64_t)blockIdx.x < ntrips) fetch(blockIdx.x);
    for (int64_t trip = blockIdx.x; trip < ntrips; trip += gridDim.x) {
        // the trip's activation chunks stay packed (16 bits per value) and are widened where they are used,
        // twice: fewer live registers, more resident wavefronts
        u32x4_t cur[LC_U];
#pragma unroll
        for (int u = 0; u < LC_U; ++u) cur[u] = nx[u];
        auto widen = [](const u32x4_t &v, float (&f)[8]) __attribute__((always_inline)) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                f[2 * d] = T::to_float((uint16_t)(v[d] & 0xffffu));
                f[2 * d + 1] = T::to_float((uint16_t)(v[d] >> 16));
            }
        };
        int lab_now[LC_U];
#pragma unroll
        for (int u = 0; u < LC_U; ++u) lab_now[u] = SHFL ? nlab[u] : 0;
        const int lab1_now = nlab1;
        if (trip + gridDim.x < ntrips) fetch(trip + gridDim.x);
        float dzr0[LC_U], dzr1[LC_U], dzr2[LC_U];        // SHFL: this thread's pixels' dz
        // One pixel's logits -> loss term and dz (the arithmetic of the loss kernel), copies on request.
        struct Dz { float d0, d1, d2, loss; };
        auto pixel = [](float z0, float z1, float z2, int lab, float w0, float w1, float w2, float scale) __attribute__((always_inline)) {
            // selects, raw v_log_f32 / v_rcp_f32 (the sum of the exponentials lies in [1, 3]): as in the loss kernel
            const bool is0 = lab == 0, is1 = lab == 1, is2 = lab == 2;
            float wl = is1 ? w1 : w0;
            wl = is2 ? w2 : wl;
            wl = (is0 | is1 | is2) ? wl : 0.f;                                          // labels outside {0,1,2}: weight 0
            const float m = fmaxf(z0, fmaxf(z1, z2));
            const float e0 = __expf(z0 - m), e1 = __expf(z1 - m), e2 = __expf(z2 - m);
            const float se = e0 + e1 + e2;
            float zl = is1 ? z1 : z2;
            zl = is0 ? z0 : zl;
            const float sw = scale * wl;
            const float gsc = sw * __builtin_amdgcn_rcpf(se);
            Dz r;
            r.d0 = fmaf(gsc, e0, is0 ? -sw : 0.f);
            r.d1 = fmaf(gsc, e1, is1 ? -sw : 0.f);
            r.d2 = fmaf(gsc, e2, is2 ? -sw : 0.f);
            r.loss = wl * ((m - zl) + 0.693147180559945f * __builtin_amdgcn_logf(se));
            return r;
        };
        // the copies of the logits and of their gradient, rounded on store, and the pixel's loss term
        auto emit = [&](int64_t pix, float z0, float z1, float z2, const Dz &r) __attribute__((always_inline)) {
            loss_sum += r.loss;
            if (a_logits) {
                a_logits[pix * 3] = T::from_float(z0);
                a_logits[pix * 3 + 1] = T::from_float(z1);
                a_logits[pix * 3 + 2] = T::from_float(z2);
            }
            if (a_dlogits) {
                a_dlogits[pix * 3] = T::from_float(r.d0);
                a_dlogits[pix * 3 + 1] = T::from_float(r.d1);
                a_dlogits[pix * 3 + 2] = T::from_float(r.d2);
            }
        };
        // ---- partial dot products of this chunk ------------------------------------
        if (SHFL) {
#pragma unroll
            for (int u = 0; u < LC_U; ++u) {
                float zz[3], xf[8];
                widen(cur[u], xf);
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    float sdot = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) sdot += xf[e] * wv[k][e];
                    zz[k] = half_wave_sum(sdot, tid & 63);       // every lane of the pixel ends with the same sum
                }
                const int64_t pix = trip * PB + u * PPI + ps;
                Dz r = pixel(zz[0], zz[1], zz[2], lab_now[u], cw0, cw1, cw2, a_scale);
                if (pix >= a_n) r = Dz{0.f, 0.f, 0.f, 0.f};
                else if (g == 0) emit(pix, zz[0], zz[1], zz[2], r);
                dzr0[u] = r.d0; dzr1[u] = r.d1; dzr2[u] = r.d2;
            }
        } else {
            if (active) {
#pragma unroll
                for (int u = 0; u < LC_U; ++u) {
                    const int q = u * PPI + ps;
                    float xf[8];
                    widen(cur[u], xf);
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
                        float sdot = 0.f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) sdot += xf[e] * wv[k][e];
                        pd[(q * 3 + k) * G + g] = sdot;
                    }
                }
            }
            __syncthreads();
            // ---- one thread per pixel: logits, loss, dz -----------------------------------
            if (tid < PB) {
                const int q = tid;
                float zz[3];
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    const float *src = pd + (q * 3 + k) * G;
                    float sdot = 0.f;
                    for (int c = 0; c < G; ++c) sdot += src[c];          // chunk order: fixed
                    zz[k] = sdot;
                }
                const int64_t pix = trip * PB + q;
                Dz r = pixel(zz[0], zz[1], zz[2], lab1_now, cw0, cw1, cw2, a_scale);
                if (pix >= a_n) r = Dz{0.f, 0.f, 0.f, 0.f};
                else emit(pix, zz[0], zz[1], zz[2], r);
                dzs[q][0] = r.d0; dzs[q][1] = r.d1; dzs[q][2] = r.d2;
            }
            __syncthreads();
        }
        // ---- this chunk of dx, and dz x^T into the running sums of dW ---------------------
        if (active) {
#pragma unroll
            for (int u = 0; u < LC_U; ++u) {
                const int q = u * PPI + ps;
                const int64_t pix = trip * PB + q;
                const float d0 = SHFL ? dzr0[u] : dzs[q][0], d1 = SHFL ? dzr1[u] : dzs[q][1], d2 = SHFL ? dzr2[u] : dzs[q][2];
                u32x4_t out;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const float a = d0 * wv[0][2 * d] + d1 * wv[1][2 * d] + d2 * wv[2][2 * d];
                    const float b = d0 * wv[0][2 * d + 1] + d1 * wv[1][2 * d + 1] + d2 * wv[2][2 * d + 1];
                    out[d] = (uint32_t)T::from_float(a) | ((uint32_t)T::from_float(b) << 16);
                }
                if (pix < a_n) __builtin_nontemporal_store(out, reinterpret_cast<u32x4_t *>(a_dx + pix * a_C + g * 8));
                float xf[8];
                widen(cur[u], xf);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    acc[0][e] += d0 * xf[e];
                    acc[1][e] += d1 * xf[e];
                    acc[2][e] += d2 * xf[e];
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
    float *out_dw = a_partial_dw + (size_t)blockIdx.x * 3 * a_C;
    for (int i = tid; i < 3 * a_C; i += LC_THREADS) {
        const int k = i / a_C, c = i - k * a_C;
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
        a_partial_loss[blockIdx.x] = s;
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
    const int G = a.C / 8;
    const bool shfl = G == 32;                           // a pixel's threads are half a wavefront
    if (is_bf16 && shfl) DLK_LAUNCH("logits_ce_kernel", (logits_ce_kernel<BF16, true>), grid, block, 0, stream, a);
    else if (is_bf16) DLK_LAUNCH("logits_ce_kernel", (logits_ce_kernel<BF16, false>), grid, block, 0, stream, a);
    else if (shfl) DLK_LAUNCH("logits_ce_kernel", (logits_ce_kernel<F16, true>), grid, block, 0, stream, a);
    else DLK_LAUNCH("logits_ce_kernel", (logits_ce_kernel<F16, false>), grid, block, 0, stream, a);
    return dlk::launch_status();
}

}  // namespace dlk
