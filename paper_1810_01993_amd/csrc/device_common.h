// Device-side building blocks shared by the gfx950 kernels: 16-bit storage
// types, fp32 -> fp16/bf16 rounding, and the 32x32x16 MFMA tile product read
// out of LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dlk {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Storage-type traits.  Tensors are handled as raw 16-bit patterns; only the
// MFMA instruction and the final rounding differ between the two types.
struct F16 {
    static __device__ __forceinline__ floatx16_t mfma(u32x4_t a, u32x4_t b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
    // 16x16 output tile, 32-deep: lane l supplies row (column) l%16, reduction elements 8*(l/16)..+7;
    // register v of lane l of the result holds row 4*(l/16) + v, column l%16
    static __device__ __forceinline__ floatx4_t mfma16(u32x4_t a, u32x4_t b, floatx4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
    // The same product accumulating in place (result registers = addend registers).  The builtin
    // leaves that choice to the register allocator, which in kernels with dozens of 4-register
    // accumulators moves them about and runs out of registers.  The compiler does not see an MFMA
    // here: the accumulator must not be touched by anything but further mfma16_acc calls until
    // mfma_acc_settle() has run.
    static __device__ __forceinline__ void mfma16_acc(floatx4_t &c, u32x4_t a, u32x4_t b) {
        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    }
    static __device__ __forceinline__ uint16_t from_float(float f) {       // nearest even
        return __builtin_bit_cast(uint16_t, (_Float16)f);
    }
    static __device__ __forceinline__ float to_float(uint16_t h) {
        return (float)__builtin_bit_cast(_Float16, h);
    }
    // two values rounded (nearest even) and packed, lo in bits 0..15: one v_cvt_pk_f16_f32
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        return __builtin_bit_cast(uint32_t, half2_t{(_Float16)lo, (_Float16)hi});
    }
};

struct BF16 {
    static __device__ __forceinline__ floatx16_t mfma(u32x4_t a, u32x4_t b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx4_t mfma16(u32x4_t a, u32x4_t b, floatx4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ void mfma16_acc(floatx4_t &c, u32x4_t a, u32x4_t b) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    }
    static __device__ __forceinline__ uint16_t from_float(float f) {       // nearest even
        uint32_t u = __builtin_bit_cast(uint32_t, f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // quiet NaN
        u += 0x7fffu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    static __device__ __forceinline__ float to_float(uint16_t h) {
        return __builtin_bit_cast(float, (uint32_t)h << 16);
    }
    // two values rounded (nearest even) and packed, lo in bits 0..15: one v_cvt_pk_bf16_f32
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        return __builtin_bit_cast(uint32_t, bf16x2_t{(__bf16)lo, (__bf16)hi});
    }
};

// Between the last mfma16_acc and the first other use of its accumulators: the result of an
// 8-pass MFMA may be read by other instruction classes only 11 or more issue slots later, a gap
// the compiler keeps for its own MFMAs and cannot keep for inline assembly.
__device__ __forceinline__ void mfma_acc_settle()
{
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// Point-wise tail of the forward convolution (bias per output column, then ReLU), applied to
// the fp32 sums before they are rounded.  bias and relu are kernel arguments (uniform).
__device__ __forceinline__ float apply_tail(float v, const float *bias, int relu, int col)
{
    if (bias) v += bias[col];
    return relu ? fmaxf(v, 0.f) : v;
}
// four consecutive columns col .. col+3 of which those below ncols exist
__device__ __forceinline__ floatx4_t apply_tail4(floatx4_t c, const float *bias, int relu, int col, int ncols)
{
    if (bias) {
        if (col + 3 < ncols && ((reinterpret_cast<uintptr_t>(bias + col) & 15) == 0)) {
            const floatx4_t b = *reinterpret_cast<const floatx4_t *>(bias + col);
            c += b;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < ncols) c[e] += bias[col + e];
        }
    }
    if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = fmaxf(c[e], 0.f);
    }
    return c;
}

// c += resid[off .. off+3] (four consecutive columns col .. col+3 of one output row, those below ncols exist)
template <class T>
__device__ __forceinline__ floatx4_t add_resid4(floatx4_t c, const uint16_t *resid, size_t off, int col, int ncols)
{
    if (col + 3 < ncols && ((reinterpret_cast<uintptr_t>(resid + off) & 7) == 0)) {
        const u32x2_t v = *reinterpret_cast<const u32x2_t *>(resid + off);
        c[0] += T::to_float((uint16_t)(v[0] & 0xffffu));
        c[1] += T::to_float((uint16_t)(v[0] >> 16));
        c[2] += T::to_float((uint16_t)(v[1] & 0xffffu));
        c[3] += T::to_float((uint16_t)(v[1] >> 16));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < ncols) c[e] += T::to_float(resid[off + e]);
    }
    return c;
}

// LDS tiles are [rows][BKT] 16-bit elements (BKT = 32 or 64) with the row
// pitch padded by 8 elements (16 bytes): pitch/16 is then odd, so the 16-byte
// fragment reads of 8 consecutive rows fall into 8 different 16-byte bank groups.
constexpr int BK = 32;
constexpr int LDS_PITCH = BK + 8;

// One BKT-deep step of the block tile product.  The wave owns TM x TN MFMA
// tiles of 32x32; sa / sb point at the wave's first row in the current LDS
// buffers.  Operand layout of v_mfma_f32_32x32x16: lane l supplies row
// (l % 32), reduction elements 8*(l / 32) .. +7 of each 16-deep slice.
template <class T, int TM, int TN, int BKT = BK>
__device__ __forceinline__ void mma_step(const uint16_t *sa, const uint16_t *sb, int lane,
                                         floatx16_t (&acc)[TM][TN])
{
    constexpr int PITCH = BKT + 8;
    const int frag = (lane & 31) * PITCH + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BKT / 16; ++ks) {
        u32x4_t a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            a[i] = *reinterpret_cast<const u32x4_t *>(sa + i * 32 * PITCH + frag + ks * 16);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            b[j] = *reinterpret_cast<const u32x4_t *>(sb + j * 32 * PITCH + frag + ks * 16);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = T::mfma(a[i], b[j], acc[i][j]);
    }
}

// Buffer resource over a dense tensor: loads whose byte offset lies at or
// beyond `bytes` return zero instead of touching memory, which is how zero
// padding and ragged tile edges are fetched without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
constexpr uint32_t OOB_OFFSET = 0xFFFFFF00u;      // beyond any tensor the boundary accepts

__device__ __forceinline__ u32x4_t buffer_load_16B(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
}

typedef int32_t i32x4_t __attribute__((ext_vector_type(4)));

// LDS byte address of a __shared__ object.
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void *)p);
}

// One direct-to-LDS load: every lane fetches 16 bytes at `byte_off` of the
// buffer `rsrc` (zero if out of range) and the wave deposits them at LDS
// address lds_base + 16*lane.  Written as inline assembly so that the
// compiler's wait-count insertion does not treat every later LDS read as
// dependent on it; completion is awaited explicitly before the barrier.
__device__ __forceinline__ void dma_load_16B(i32x4_t rsrc, uint32_t lds_base, uint32_t byte_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(byte_off), "s"(rsrc)
                 : "memory", "m0");
}

__device__ __forceinline__ i32x4_t make_rsrc_words(const void *base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)(uintptr_t)base;
    i32x4_t r;
    r[0] = (int32_t)(uint32_t)a;
    r[1] = (int32_t)((uint32_t)(a >> 32) & 0xffffu);     // stride 0: raw buffer
    r[2] = (int32_t)bytes;
    r[3] = 0x00020000;
    return r;
}

// Accumulator layout of a 32x32 MFMA tile: register v of lane l holds
// row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Spread consecutive workgroup ids over the 8 XCDs so that each XCD (own L2)
// works through one contiguous run of tiles.  Workgroups are dealt to XCDs
// round-robin by id; this maps id -> tile so that XCD x gets tiles
// [x*n/8, (x+1)*n/8).
__device__ __forceinline__ int xcd_remap(int bid, int nblocks)
{
    constexpr int XCDS = 8;
    const int per = nblocks / XCDS, rem = nblocks % XCDS;
    const int xcd = bid % XCDS, slot = bid / XCDS;
    // XCDs [0, rem) own per+1 tiles, the rest own per tiles
    const int start = xcd * per + (xcd < rem ? xcd : rem);
    return start + slot;
}

}  // namespace dlk
