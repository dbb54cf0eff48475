// Shared device-side types and helpers of the bf16 (matrix-core) kernels.
//
// MFMA used everywhere: v_mfma_f32_16x16x32_bf16, D[16x16] += A[16x32] * B[32x16].
// Lane l of the wavefront holds
//   A: row m = l % 16, the 8 values k = 8*(l/16) .. 8*(l/16)+7
//   B: column n = l % 16, the 8 values k = 8*(l/16) .. 8*(l/16)+7
//   D: column n = l % 16, the 4 rows m = 4*(l/16) .. 4*(l/16)+3
// All kernels put the WEIGHTS in A (m = output feature / channel) and the
// ACTIVATIONS in B (n = batch row or pixel), so a lane ends up holding four
// consecutive output channels of one pixel: one packed 8-byte NHWC store.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace seedinf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even.  Written as two 2-wide vector conversions so that each becomes one packed
// hardware conversion (v_cvt_pk_bf16_f32); element-wise casts, and a 4-wide conversion whose result is then
// reinterpreted as integers, cost a conversion and a byte permute per element.
__device__ __forceinline__ bf16x4 to_bf16x4(floatx4 v)
{
    const bf16x2 lo = __builtin_convertvector((floatx2){v[0], v[1]}, bf16x2);
    const bf16x2 hi = __builtin_convertvector((floatx2){v[2], v[3]}, bf16x2);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
}

__device__ __forceinline__ floatx4 relu4(floatx4 v)
{
    floatx4 r;
    r[0] = fmaxf(v[0], 0.0f); r[1] = fmaxf(v[1], 0.0f); r[2] = fmaxf(v[2], 0.0f); r[3] = fmaxf(v[3], 0.0f);
    return r;
}

// ReLU on four packed bf16 values: as signed 16-bit integers every negative float is negative
// and every non-negative float is non-negative, so max(x, 0) per 16-bit lane is exact (one v_pk_max_i16
// per pair).
typedef short shortx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x4 relu_bf16x4(bf16x4 v)
{
    const shortx2 z = {0, 0};
    const bf16x2 lo = __builtin_shufflevector(v, v, 0, 1), hi = __builtin_shufflevector(v, v, 2, 3);
    const shortx2 l = __builtin_elementwise_max(__builtin_bit_cast(shortx2, lo), z);
    const shortx2 h = __builtin_elementwise_max(__builtin_bit_cast(shortx2, hi), z);
    return __builtin_shufflevector(__builtin_bit_cast(bf16x2, l), __builtin_bit_cast(bf16x2, h), 0, 1, 2, 3);
}

__device__ __forceinline__ floatx4 to_floatx4(bf16x4 v) { return __builtin_convertvector(v, floatx4); }

__device__ __forceinline__ floatx4 max4(floatx4 a, floatx4 b)
{
    floatx4 r;
    r[0] = fmaxf(a[0], b[0]); r[1] = fmaxf(a[1], b[1]); r[2] = fmaxf(a[2], b[2]); r[3] = fmaxf(a[3], b[3]);
    return r;
}

// (row, column) of an index that advances by a fixed step through a row-major region `rw` wide: one division at the
// start, then adds (the step's row and column parts are uniform).  The staging and pooling loops of the
// layer-by-layer kernels walk their regions with it: a division per item was a large part of their instructions.
struct RowWalk {
    int r, c, dr, dc, rw;
    __device__ __forceinline__ RowWalk(int first, int step, int width) : rw(width)
    {
        r = first / width; c = first - r * width;
        dr = step / width; dc = step - dr * width;
    }
    __device__ __forceinline__ void next()
    {
        c += dc; r += dr;
        if (c >= rw) { c -= rw; ++r; }
    }
};

// Maximum of two bf16 pairs with the packed fp16 maximum.  bf16 and fp16 are both sign-magnitude, so of two bit
// patterns that are finite numbers in both formats (as bf16: |x| < 2^121, far beyond any activation) the larger
// fp16 is the larger bf16, and the instruction returns that operand bit for bit (half-denormals included: the
// fp16 denormal mode of these kernels keeps them).  Four times fewer instructions than widening to fp32.
__device__ __forceinline__ uint32_t bf16x2_max(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
// the padding value of such maxima, as a pair: the most negative pattern that is finite as fp16 (-2.6e36 as bf16)
constexpr uint32_t BF16X2_LOWEST = 0xFBFFFBFFu;
__device__ __forceinline__ uint4 bf16x8_max(uint4 a, uint4 b)
{
    return uint4{bf16x2_max(a.x, b.x), bf16x2_max(a.y, b.y), bf16x2_max(a.z, b.z), bf16x2_max(a.w, b.w)};
}
// the two bf16 of a pair as fp32
__device__ __forceinline__ float bf16_lo_f32(uint32_t v) { return __builtin_bit_cast(float, v << 16); }
__device__ __forceinline__ float bf16_hi_f32(uint32_t v) { return __builtin_bit_cast(float, v & 0xffff0000u); }

// 8 fp32 -> 8 bf16 (round to nearest even, the hardware conversion)
__device__ __forceinline__ bf16x8 to_bf16x8(floatx4 lo, floatx4 hi)
{
    const bf16x4 a = to_bf16x4(lo), b = to_bf16x4(hi);
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// 8 bytes (two dwords, little endian) -> 8 bf16 holding the integers 0..255 exactly
__device__ __forceinline__ bf16x8 u8x8_to_bf16x8(uint32_t lo, uint32_t hi)
{
    const floatx4 a = {(float)(lo & 0xff), (float)((lo >> 8) & 0xff), (float)((lo >> 16) & 0xff), (float)(lo >> 24)};
    const floatx4 b = {(float)(hi & 0xff), (float)((hi >> 8) & 0xff), (float)((hi >> 16) & 0xff), (float)(hi >> 24)};
    return to_bf16x8(a, b);
}

// Asynchronous global -> LDS load (no registers): lane l's 16 bytes land at (wave-uniform LDS base in M0) +
// 16 * l.  Written as inline assembly because the compiler would otherwise wait for it before the next LDS
// access of any kind; stage_wait() collects every such load the wavefront has issued.
__device__ __forceinline__ void g2lds16(const void* gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void stage_wait()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace seedinf
