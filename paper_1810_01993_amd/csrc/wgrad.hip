// Filter-gradient kernel for gfx950.
//
// GEMM view: rows = output channel k, columns j = (r*S + s)*C + c, reduction
// over the N*P*Q output pixels.  Both operands are stored channel-contiguous
// (NHWC) while the MFMA wants 8 consecutive reduction elements (pixels) per
// lane, so tiles are transposed on their way into LDS: a thread loads the
// same 8 channels of 4 consecutive pixels, regroups them in registers into
// 8 x (4 pixels) and writes 8-byte pieces into a [channel][pixel] LDS tile.
// The pixel range is cut into `splits` slices (grid.y); every slice writes an
// fp32 partial tile, and a second kernel adds the slices in a fixed order.
#include <cstdint>
#include <cstdlib>
#include "device_common.h"
#include "kernels.h"

namespace dlk {

struct PixelCursor {          // (n, p, q) of one output pixel, advanced without division
    int n, p, q;
    __device__ __forceinline__ void init(int pix, int P, int Q) {
        n = pix / (P * Q);
        const int rem = pix - n * (P * Q);
        p = rem / Q;
        q = rem - p * Q;
    }
    __device__ __forceinline__ void advance(int by, int P, int Q) {
        q += by;
        while (q >= Q) {
            q -= Q;
            if (++p == P) { p = 0; ++n; }
        }
    }
};

template <class T, int BM, int BN, int WM, int WN, bool VECA, bool VECB>
__global__ __launch_bounds__(WM *WN * 64) void wgrad_kernel(const WgradArgs p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int PG = 4;                              // pixels regrouped per thread item
    constexpr int ITEMS_A = (BM / 8) * (BK / PG), ITEMS_B = (BN / 8) * (BK / PG);
    constexpr int IA = (ITEMS_A + NT - 1) / NT, IB = (ITEMS_B + NT - 1) / NT;

    extern __shared__ __align__(16) uint16_t lds[];
    uint16_t *sA = lds;                                // [2][BM][LDS_PITCH]   dy^T : [k][pixel]
    uint16_t *sB = lds + 2 * BM * LDS_PITCH;           // [2][BN][LDS_PITCH]   x^T  : [j][pixel]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int RSC = p.R * p.S * p.C;
    const int npix = p.N * p.P * p.Q;
    const int tiles_n = (RSC + BN - 1) / BN;
    const int k0 = (blockIdx.x / tiles_n) * BM, j0 = (blockIdx.x % tiles_n) * BN;
    const int pix_begin = blockIdx.y * p.chunk;
    const int pix_end = min(npix, pix_begin + p.chunk);

    // ---- item coordinates --------------------------------------------------
    // item -> (cv = 8-channel column group, pg = group of 4 consecutive pixels)
    int b_ih[IB], b_iw[IB], b_c[IB];                   // tap offset and channel of the item's columns
    bool b_col_ok[IB];
    PixelCursor cur[IB];
#pragma unroll
    for (int it = 0; it < IB; ++it) {
        const int item = tid + it * NT;
        const int cv = item % (BN / 8), pg = item / (BN / 8);
        const int j = j0 + cv * 8;
        b_col_ok[it] = item < ITEMS_B && j < RSC;
        const int tap = j / p.C;
        b_c[it] = j - tap * p.C;
        const int r = tap / p.S, s = tap - r * p.S;
        b_ih[it] = r * p.dh - p.ph;
        b_iw[it] = s * p.dw - p.pw;
        cur[it].init(pix_begin + pg * PG, p.P, p.Q);
    }

    u32x4_t ra[IA][PG], rb[IB][PG];
    int pix_base = pix_begin;                          // first pixel of the block being loaded

    auto load_tiles = [&]() {
#pragma unroll
        for (int it = 0; it < IA; ++it) {
            const int item = tid + it * NT;
            const int cv = item % (BM / 8), pg = item / (BM / 8);
            const int k = k0 + cv * 8;
#pragma unroll
            for (int g = 0; g < PG; ++g) {
                const int pix = pix_base + pg * PG + g;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (item < ITEMS_A && pix < pix_end) {
                    if constexpr (VECA) {
                        if (k < p.K) v = *reinterpret_cast<const u32x4_t *>(p.dy + (size_t)pix * p.K + k);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const uint32_t h = (k + e < p.K) ? p.dy[(size_t)pix * p.K + k + e] : 0u;
                            v[e >> 1] |= h << (16 * (e & 1));
                        }
                    }
                }
                ra[it][g] = v;
            }
        }
#pragma unroll
        for (int it = 0; it < IB; ++it) {
            const int item = tid + it * NT;
            const int pg = item / (BN / 8);
            PixelCursor pc = cur[it];
#pragma unroll
            for (int g = 0; g < PG; ++g) {
                const int pix = pix_base + pg * PG + g;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (b_col_ok[it] && pix < pix_end) {
                    if constexpr (VECB) {
                        const int ih = pc.p * p.sh + b_ih[it], iw = pc.q * p.sw + b_iw[it];
                        if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                            v = *reinterpret_cast<const u32x4_t *>(
                                p.x + (size_t)((pc.n * p.H + ih) * p.W + iw) * p.C + b_c[it]);
                    } else {
                        const int cv = item % (BN / 8);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int j = j0 + cv * 8 + e;
                            uint32_t h = 0u;
                            if (j < RSC) {
                                const int tap = j / p.C, c = j - tap * p.C;
                                const int r = tap / p.S, s = tap - r * p.S;
                                const int ih = pc.p * p.sh - p.ph + r * p.dh, iw = pc.q * p.sw - p.pw + s * p.dw;
                                if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                                    h = p.x[(size_t)((pc.n * p.H + ih) * p.W + iw) * p.C + c];
                            }
                            v[e >> 1] |= h << (16 * (e & 1));
                        }
                    }
                }
                rb[it][g] = v;
                pc.advance(1, p.P, p.Q);
            }
            cur[it].advance(BK, p.P, p.Q);
        }
        pix_base += BK;
    };

    // [4 pixels][8 channels] -> [8 channels][4 pixels], 8-byte LDS writes
    auto store_transposed = [&](uint16_t *dst_tile, const u32x4_t (&r)[PG], int cv, int pg) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            u32x2_t lo, hi;                             // channel 2d and channel 2d+1
            lo[0] = (r[0][d] & 0xffffu) | (r[1][d] << 16);
            lo[1] = (r[2][d] & 0xffffu) | (r[3][d] << 16);
            hi[0] = (r[0][d] >> 16) | (r[1][d] & 0xffff0000u);
            hi[1] = (r[2][d] >> 16) | (r[3][d] & 0xffff0000u);
            *reinterpret_cast<u32x2_t *>(dst_tile + (cv * 8 + 2 * d) * LDS_PITCH + pg * PG) = lo;
            *reinterpret_cast<u32x2_t *>(dst_tile + (cv * 8 + 2 * d + 1) * LDS_PITCH + pg * PG) = hi;
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int it = 0; it < IA; ++it) {
            const int item = tid + it * NT;
            if (item < ITEMS_A) store_transposed(sA + buf * BM * LDS_PITCH, ra[it], item % (BM / 8), item / (BM / 8));
        }
#pragma unroll
        for (int it = 0; it < IB; ++it) {
            const int item = tid + it * NT;
            if (item < ITEMS_B) store_transposed(sB + buf * BN * LDS_PITCH, rb[it], item % (BN / 8), item / (BN / 8));
        }
    };

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = pix_end > pix_begin ? (pix_end - pix_begin + BK - 1) / BK : 0;
    if (nk > 0) {
        load_tiles();
        store_tiles(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cb = kt & 1;
            if (kt + 1 < nk) load_tiles();
            mma_step<T, TM, TN, BK>(sA + cb * BM * LDS_PITCH + wm * TM * 32 * LDS_PITCH,
                                sB + cb * BN * LDS_PITCH + wn * TN * 32 * LDS_PITCH, lane, acc);
            if (kt + 1 < nk) store_tiles(cb ^ 1);
            __syncthreads();
        }
    }

    float *out = p.partial + (size_t)blockIdx.y * p.K * RSC;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + (wm * TM + i) * 32 + acc_row(v, lane);
            if (k >= p.K) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = j0 + (wn * TN + j) * 32 + (lane & 31);
                if (col < RSC) out[(size_t)k * RSC + col] = acc[i][j][v];
            }
        }
}

template <class T, int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const WgradArgs &a, hipStream_t stream)
{
    const int RSC = a.R * a.S * a.C;
    const int64_t tiles = (int64_t)((a.K + BM - 1) / BM) * ((RSC + BN - 1) / BN);
    constexpr size_t lds = size_t(2) * (BM + BN) * LDS_PITCH * sizeof(uint16_t);
    static_assert(lds <= 64 * 1024, "needs the dynamic LDS attribute");
    const dim3 grid((unsigned)tiles, (unsigned)a.splits), block(WM * WN * 64);
    const bool va = a.K % 8 == 0, vb = a.C % 8 == 0;
    if (va && vb)
        DLK_LAUNCH(kname("wgrad_kernel", {BM, BN}), (wgrad_kernel<T, BM, BN, WM, WN, true, true>), grid, block, lds, stream, a);
    else if (vb)
        DLK_LAUNCH(kname("wgrad_kernel", {BM, BN}), (wgrad_kernel<T, BM, BN, WM, WN, false, true>), grid, block, lds, stream, a);
    else if (va)
        DLK_LAUNCH(kname("wgrad_kernel", {BM, BN}), (wgrad_kernel<T, BM, BN, WM, WN, true, false>), grid, block, lds, stream, a);
    else
        DLK_LAUNCH(kname("wgrad_kernel", {BM, BN}), (wgrad_kernel<T, BM, BN, WM, WN, false, false>), grid, block, lds, stream, a);
    return dlk::launch_status();
}

hipError_t launch_wgrad(const WgradArgs &a, bool is_bf16, hipStream_t stream)
{
    return is_bf16 ? launch_cfg<BF16, 128, 128, 2, 2>(a, stream) : launch_cfg<F16, 128, 128, 2, 2>(a, stream);
}

// ---- ordered reduction of the split partials ------------------------------
// Workgroup = XW outputs x G slice groups (XW * G = 256).  Thread (x, g) adds
// slices g, g+G, g+2G, ... in ascending order with four independent running
// sums (so that several loads are in flight), combines them in a fixed order,
// and the G groups are then added in ascending g through LDS: the summation
// tree depends only on `splits` and G, never on timing.  G = 4 in general;
// G = 32 for the few-outputs, many-slices case (the thin filter gradient:
// 768 outputs x 2048 slices), where 4 groups would leave each thread a chain
// of 128 dependent round trips.
template <int OUT, int G>   // OUT: 0 f16, 1 bf16, 2 f32
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int splits, int64_t n,
                                                            void *out, const float *__restrict__ bias, int relu, int ncols,
                                                            const uint16_t *__restrict__ resid)
{
    constexpr int XW = 256 / G;
    __shared__ float part[G][XW];
    const int x = threadIdx.x % XW, g = threadIdx.x / XW;
    for (int64_t base = (int64_t)blockIdx.x * XW; base < n; base += (int64_t)gridDim.x * XW) {
        const int64_t i = base + x;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        if (i < n) {
            int z = g;
            for (; z + 3 * G < splits; z += 4 * G) {
                s0 += partial[(size_t)z * n + i];
                s1 += partial[(size_t)(z + G) * n + i];
                s2 += partial[(size_t)(z + 2 * G) * n + i];
                s3 += partial[(size_t)(z + 3 * G) * n + i];
            }
            for (; z < splits; z += G) s0 += partial[(size_t)z * n + i];
        }
        part[g][x] = (s0 + s1) + (s2 + s3);
        __syncthreads();
        if (g == 0 && i < n) {
            float s;
            if constexpr (G == 4) {
                s = (part[0][x] + part[1][x]) + (part[2][x] + part[3][x]);
            } else {
                s = 0.f;
#pragma unroll
                for (int q = 0; q < G; q += 4) s += (part[q][x] + part[q + 1][x]) + (part[q + 2][x] + part[q + 3][x]);
            }
            if (OUT != 2 && resid) s += OUT == 1 ? BF16::to_float(resid[i]) : F16::to_float(resid[i]);   // same layout and type as out
            if (bias || relu) s = apply_tail(s, bias, relu, (int)(i % ncols));
            if constexpr (OUT == 0) reinterpret_cast<uint16_t *>(out)[i] = F16::from_float(s);
            else if constexpr (OUT == 1) reinterpret_cast<uint16_t *>(out)[i] = BF16::from_float(s);
            else reinterpret_cast<float *>(out)[i] = s;
        }
        __syncthreads();
    }
}

// The G = 4 reduction with four consecutive outputs per thread (16-byte loads of the partial sums, n % 4 == 0):
// every output is summed in exactly the order of the kernel above, so the two give identical bits.
template <int OUT>
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const float *__restrict__ partial, int splits, int64_t n,
                                                             void *out, const float *__restrict__ bias, int relu, int ncols,
                                                             const uint16_t *__restrict__ resid)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ f4 part[4][64];
    const int x = threadIdx.x & 63, g = threadIdx.x >> 6;
    for (int64_t base = (int64_t)blockIdx.x * 256; base < n; base += (int64_t)gridDim.x * 256) {
        const int64_t i = base + 4 * x;
        f4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
        if (i < n) {
            int z = g;
            for (; z + 12 < splits; z += 16) {
                s0 += *reinterpret_cast<const f4 *>(partial + (size_t)z * n + i);
                s1 += *reinterpret_cast<const f4 *>(partial + (size_t)(z + 4) * n + i);
                s2 += *reinterpret_cast<const f4 *>(partial + (size_t)(z + 8) * n + i);
                s3 += *reinterpret_cast<const f4 *>(partial + (size_t)(z + 12) * n + i);
            }
            for (; z < splits; z += 4) s0 += *reinterpret_cast<const f4 *>(partial + (size_t)z * n + i);
        }
        part[g][x] = (s0 + s1) + (s2 + s3);
        __syncthreads();
        if (g == 0 && i < n) {
            const f4 v = (part[0][x] + part[1][x]) + (part[2][x] + part[3][x]);
            float s[4] = {v[0], v[1], v[2], v[3]};
            if (OUT != 2 && resid) {
                const uint2 rv = *reinterpret_cast<const uint2 *>(resid + i);
                const uint16_t r[4] = {(uint16_t)(rv.x & 0xffffu), (uint16_t)(rv.x >> 16), (uint16_t)(rv.y & 0xffffu), (uint16_t)(rv.y >> 16)};
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] += OUT == 1 ? BF16::to_float(r[e]) : F16::to_float(r[e]);
            }
            if (bias || relu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] = apply_tail(s[e], bias, relu, (int)((i + e) % ncols));
            }
            if constexpr (OUT == 2) {
                *reinterpret_cast<f4 *>(reinterpret_cast<float *>(out) + i) = f4{s[0], s[1], s[2], s[3]};
            } else {
                uint16_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = OUT == 1 ? BF16::from_float(s[e]) : F16::from_float(s[e]);
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + i) =
                    uint2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
            }
        }
        __syncthreads();
    }
}

static hipError_t launch_reduce4(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype, const float *bias,
                                 int32_t relu, int32_t ncols, const uint16_t *resid, hipStream_t stream)
{
    const int64_t want = (n + 255) / 256;
    const dim3 grid((unsigned)(want < 16384 ? want : 16384)), block(256);
    if (out_dtype == 0)
        DLK_LAUNCH("splitk_reduce4_kernel", splitk_reduce4_kernel<0>, grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, resid);
    else if (out_dtype == 1)
        DLK_LAUNCH("splitk_reduce4_kernel", splitk_reduce4_kernel<1>, grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, resid);
    else
        DLK_LAUNCH("splitk_reduce4_kernel", splitk_reduce4_kernel<2>, grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, nullptr);
    return dlk::launch_status();
}

template <int G>
static hipError_t launch_reduce_g(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype, const float *bias,
                                  int32_t relu, int32_t ncols, const uint16_t *resid, hipStream_t stream)
{
    constexpr int XW = 256 / G;
    const int64_t want = (n + XW - 1) / XW;
    const dim3 grid((unsigned)(want < 16384 ? want : 16384)), block(256);
    if (out_dtype == 0)
        DLK_LAUNCH(kname("splitk_reduce_kernel", {G}), (splitk_reduce_kernel<0, G>), grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, resid);
    else if (out_dtype == 1)
        DLK_LAUNCH(kname("splitk_reduce_kernel", {G}), (splitk_reduce_kernel<1, G>), grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, resid);
    else
        DLK_LAUNCH(kname("splitk_reduce_kernel", {G}), (splitk_reduce_kernel<2, G>), grid, block, 0, stream, partial, splits, n, out, bias, relu, ncols, nullptr);
    return dlk::launch_status();
}

hipError_t launch_splitk_reduce_tail(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype,
                                     const float *bias, int32_t relu, int32_t ncols, const uint16_t *resid, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    if (ncols < 1 || (resid && out_dtype == 2)) return hipErrorInvalidValue;
    if (splits >= 128 && n <= 8192) return launch_reduce_g<32>(partial, splits, n, out, out_dtype, bias, relu, ncols, resid, stream);
    static const int vec = tuning_knob("DLCONV_REDUCE4", 1); // tuning override: 0 = one output per thread always
    const bool aligned = (reinterpret_cast<uintptr_t>(partial) % 16 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(resid) % 8 == 0);
    if (vec && n % 4 == 0 && n >= 65536 && aligned)
        return launch_reduce4(partial, splits, n, out, out_dtype, bias, relu, ncols, resid, stream);
    return launch_reduce_g<4>(partial, splits, n, out, out_dtype, bias, relu, ncols, resid, stream);
}

hipError_t launch_splitk_reduce(const float *partial, int32_t splits, int64_t n, void *out, int out_dtype,
                                hipStream_t stream)
{
    return launch_splitk_reduce_tail(partial, splits, n, out, out_dtype, nullptr, 0, 1, nullptr, stream);
}

}  // namespace dlk
