// Element types of the attention kernels.  The pool, Q and the output hold 16-bit floats:
// bf16 (the default) or IEEE half (the precision the paper's system served in, Sec. 6.1).
// Everything that depends on which -- the matrix instructions, the conversion from fp32, the
// widening back, the bit pattern of 1.0 -- is collected here; the copies (append, gather,
// restore) only move 16-bit words and do not care.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cs {

typedef uint32_t e_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t e_u32x2 __attribute__((ext_vector_type(2)));
typedef float e_f32x4 __attribute__((ext_vector_type(4)));

struct Bf16 {
    typedef __bf16 x8 __attribute__((ext_vector_type(8)));
    typedef short s4 __attribute__((ext_vector_type(4)));
    typedef __bf16 x2 __attribute__((ext_vector_type(2)));
    static constexpr uint32_t kOnes = 0x3f803f80u;                 // two 1.0
    // 16x16 tile, 32 values of the contraction per call: A and B hold 8 values per lane
    static __device__ __forceinline__ e_f32x4 mfma32(e_u32x4 a, e_u32x4 b, e_f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(x8, a), __builtin_bit_cast(x8, b), c, 0, 0, 0);
    }
    // 16 values of the contraction per call: 4 values per lane
    static __device__ __forceinline__ e_f32x4 mfma16(e_u32x2 a, e_u32x2 b, e_f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s4, a), __builtin_bit_cast(s4, b), c, 0, 0, 0);
    }
    // two floats -> one dword, round to nearest even
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        x2 v = { (__bf16)lo, (__bf16)hi };
        return __builtin_bit_cast(uint32_t, v);
    }
    // exact sum of the two values of a dword
    static __device__ __forceinline__ float sum2(uint32_t w) {
        return __builtin_bit_cast(float, w << 16) + __builtin_bit_cast(float, w & 0xffff0000u);
    }
    // Whether the prefill kernel may scale Q once (by the softmax scale, rounded back to the
    // element type) instead of scaling every score: bf16's 8 mantissa bits do not stand the
    // second rounding on peaked softmaxes (max error 3e-2 to 8e-2 with queries scaled by 4-10).
    static constexpr bool kScaleFoldsIntoQ = false;
    static __device__ __forceinline__ uint32_t scale2(uint32_t w, float f) {
        return pack(__builtin_bit_cast(float, w << 16) * f, __builtin_bit_cast(float, w & 0xffff0000u) * f);
    }
};

struct F16 {
    typedef _Float16 x8 __attribute__((ext_vector_type(8)));
    typedef _Float16 x4 __attribute__((ext_vector_type(4)));
    typedef _Float16 x2 __attribute__((ext_vector_type(2)));
    static constexpr uint32_t kOnes = 0x3c003c00u;
    static __device__ __forceinline__ e_f32x4 mfma32(e_u32x4 a, e_u32x4 b, e_f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(x8, a), __builtin_bit_cast(x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ e_f32x4 mfma16(e_u32x2 a, e_u32x2 b, e_f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(x4, a), __builtin_bit_cast(x4, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        x2 v = { (_Float16)lo, (_Float16)hi };
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ float sum2(uint32_t w) {
        const x2 v = __builtin_bit_cast(x2, w);
        return (float)v[0] + (float)v[1];
    }
    // 11 mantissa bits stand it (max error 6e-3 with queries scaled by 6; one vector instruction
    // less per score)
    static constexpr bool kScaleFoldsIntoQ = true;
    static __device__ __forceinline__ uint32_t scale2(uint32_t w, float f) {
        const x2 v = __builtin_bit_cast(x2, w);
        return pack((float)v[0] * f, (float)v[1] * f);
    }
};

}  // namespace cs
