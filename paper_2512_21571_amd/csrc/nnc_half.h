// The two 16-bit storage formats of weights, cache rows and matrix-core operands: bf16 and IEEE
// binary16 (the paper's "F16", Section 4, experimental setup).  Kernels take one of these
// structs as a template argument; everything format-specific (rounding, widening, packing, the
// matrix-core instruction) goes through it, so both formats share every kernel body.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nnc {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_v __attribute__((ext_vector_type(4)));

// Element type of a model: what the launchers dispatch on.
enum Dtype { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };

struct Bf16 {
  static constexpr int kDtype = DT_BF16;
  static constexpr bool kW8 = false;  // the weights of a GEMM are in this format too
  // A small value keeps fewer and fewer significant bits below the smallest normal number;
  // bf16 has the exponent range of fp32, so operands need no scaling before they are split.
  static constexpr bool kNarrowRange = false;
  static constexpr uint32_t kOnes2 = 0x3f803f80u;  // (1.0, 1.0)
  typedef __bf16 vec8 __attribute__((ext_vector_type(8)));
  typedef __bf16 vec2 __attribute__((ext_vector_type(2)));
  typedef float fvec2 __attribute__((ext_vector_type(2)));
  // fp32 -> 16 stored bits, round to nearest, ties to even; NaN stays NaN.
  static __device__ __forceinline__ uint32_t bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
  }
  static __device__ __forceinline__ float widen(uint32_t b) { return __uint_as_float(b << 16); }
  // two values in one word, low half = a (the hardware conversion: same bits as bits() for every non-NaN)
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(fvec2{a, b}, vec2));
  }
  static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
  static __device__ __forceinline__ f32x4_t mfma(u32x4_v a, u32x4_v b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0, 0);
  }
};

struct Fp16 {
  static constexpr int kDtype = DT_F16;
  static constexpr bool kW8 = false;
  // binary16 normals end at 2^-14: an operand vector of small magnitude (an embedding row is
  // ~0.02) must be brought to unit scale before it is split into pieces.
  static constexpr bool kNarrowRange = true;
  static constexpr uint32_t kOnes2 = 0x3c003c00u;
  typedef _Float16 vec8 __attribute__((ext_vector_type(8)));
  typedef _Float16 vec2 __attribute__((ext_vector_type(2)));
  typedef float fvec2 __attribute__((ext_vector_type(2)));
  // the hardware conversion rounds to nearest even, keeps subnormals, overflows to infinity
  static __device__ __forceinline__ uint32_t bits(float f) {
    // What is converted is the value as rounded to fp32.  Left visible, a product that made f is
    // folded into the conversion (v_fma_mixlo_f16: one rounding of the exact product instead of
    // two) for some elements of an unrolled loop and not for others, differently in every
    // instantiation, and kernels that promise the same bits stop agreeing.
    asm("" : "+v"(f));
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
  }
  static __device__ __forceinline__ float widen(uint32_t b) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)b);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) { return bits(a) | (bits(b) << 16); }
  static __device__ __forceinline__ float lo(uint32_t w) { return widen(w & 0xffffu); }
  static __device__ __forceinline__ float hi(uint32_t w) { return widen(w >> 16); }
  static __device__ __forceinline__ f32x4_t mfma(u32x4_v a, u32x4_v b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0, 0);
  }
};

// bf16 activations and matrix-core products, weights stored as signed bytes with one fp32 scale
// per output row (weight-only 8-bit): a byte is widened to bf16 exactly (|q| <= 127 needs 7 bits)
// right before the product, the scale multiplies the row's sum in the epilogue.
struct Bf16W8 : Bf16 {
  static constexpr bool kW8 = true;
  // 8 signed bytes (two words) -> 8 bf16 in operand order
  static __device__ __forceinline__ u32x4_v widen8(uint32_t lo, uint32_t hi) {
    auto two = [](uint32_t w, int sh) __attribute__((always_inline)) {
      const float a = (float)(int)(int8_t)(w >> sh), b = (float)(int)(int8_t)(w >> (sh + 8));
      return pack2(a, b);
    };
    return u32x4_v{two(lo, 0), two(lo, 16), two(hi, 0), two(hi, 16)};
  }
};

// Split v into up to three 16-bit pieces whose sum is v to fp32 accuracy (value, rounded
// remainder, rounded remainder of that).
template <class HF>
__device__ __forceinline__ void split_pieces(float v, int nsplit, uint32_t* piece) {
  // the remainders are those of v as rounded to fp32: without this the compiler may fuse the
  // subtraction with the product that made v, in one caller and not in another
#pragma clang fp contract(off)
  float r = v;
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    if (s < nsplit) {
      const uint32_t b = HF::bits(r);
      piece[s] = b;
      r -= HF::widen(b);
    }
  }
}

}  // namespace nnc
