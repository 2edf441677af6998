// Pieces shared by the matrix-core MicroAttention kernels for 16-bit operands: operand types, the 16-byte
// streaming load, the 16 x 16 x 32 product, the high + low split of the softmax weights, the merge buffers.
#pragma once
#include <hip/hip_runtime.h>

#include "kernel_params.h"

namespace da {
namespace mfma16bit {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegInf = -__builtin_inff();
constexpr float kLn2 = 0.69314718055994530942f;
constexpr int kHeadTile = 16;  // columns per MFMA tile (N dimension)
constexpr int kChunk = 32;     // tokens per wavefront step (MFMA K dimension of the PV product)
constexpr int kWaves = 4;      // wavefronts per workgroup
// bf16 weights are taken against a reference maximum that follows the running maximum only when that has grown
// by more than this (base-2 units): weights stay below 2^16, well inside the range of bf16 and fp32, and the
// accumulator is rescaled a handful of times per split instead of whenever any column's maximum moves
constexpr float kLazyRescale = 16.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }

// Two floats -> packed bf16 (round to nearest even), first value in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16-byte streaming load: K and V are read exactly once, so the non-temporal hint keeps them from
// displacing anything in the caches (measurably faster than a plain load on this GPU).
__device__ __forceinline__ u32x4 load16_stream(const char *p) { return __builtin_nontemporal_load((const u32x4 *)p); }

// 16 x 16 x 32 matrix-core product of 16-bit operands with fp32 accumulation; F16: IEEE half, else bf16
template <bool F16>
__device__ __forceinline__ f32x4 mfma16(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Softmax weights go into the PV product as a high + a low 16-bit part, so that they carry about 16 (bf16) or 22
// (half) mantissa bits.  Half has a narrow exponent (numbers under 6.1e-5 lose mantissa bits, under 6e-8 they
// vanish): the kernel hands over weights relative to the chunk's own maximum (largest = 1) multiplied by 2^15
// (below the largest half, 65504), so that within a chunk weights down to 2^-29 of the largest keep their full
// precision; the chunk's product is scaled back when it is added to the accumulator.
template <bool F16>
struct Weights;
template <>
struct Weights<false> {
    static __device__ __forceinline__ void split(float a, float b, uint32_t &hi, uint32_t &lo)
    {
        hi = pack_bf16(a, b);
        lo = pack_bf16(a - as_f(hi << 16), b - as_f(hi & 0xFFFF0000u));
    }
};
template <>
struct Weights<true> {
    static constexpr float kScale = 32768.0f, kUnscale = 1.0f / 32768.0f;
    static __device__ __forceinline__ void split(float a, float b, uint32_t &hi, uint32_t &lo)
    {
        a *= kScale;
        b *= kScale;
        const fp16x2 h = __builtin_amdgcn_cvt_pkrtz(a, b);  // toward zero: the remainder is >= 0 and exact in fp32
        hi = __builtin_bit_cast(uint32_t, h);
        lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a - (float)h[0], b - (float)h[1]));
    }
};

template <int COLS>
struct MergeBuffers {
    float m[kWaves][COLS];
    float e[kWaves][COLS];
    float o[kWaves][COLS][kHeadDim];
};

}  // namespace mfma16bit
}  // namespace da
