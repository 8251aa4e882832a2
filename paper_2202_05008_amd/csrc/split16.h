// fp32-accurate products on the 16-bit matrix instruction: two-term half-precision operand splits.
//
// A value x (already multiplied by a power of two s chosen per tensor so that it sits well inside
// fp16's exponent range) is represented as x ~ h + 2^-11 m with h = fp16(x) and
// m = fp16(2^11 (x - h)): the residual is exact in fp32, at most half an ulp of h, and scaling it
// by 2^11 brings it back to the magnitude of x, so it keeps 11 significand bits of its own;
// |x - h - 2^-11 m| <= 2^-22 |x|.  A product of two such values is accumulated in fp32 as
//     h h'  (one accumulator)   and   h m' + m h'  (a second one, added with the factor 2^-11);
// every fp16 x fp16 product is exact in fp32 and the dropped m m' is below 2^-22 of the product.
//
// Two hardware facts shape the code.  (1) v_cvt_pk_f16_f32, which the compiler picks for a pair of
// conversions, returns zero where the single conversion returns a subnormal: the residual must be
// taken against the value that is actually stored, so the pair is converted once and the same
// register feeds both uses.  A leading term that came out as zero is harmless: the whole value
// then sits in m (11 bits of it), and the tensor scales keep such values below 2^-14 / s.
// (2) The leading term overflows beyond 65504 / s.  Tensors whose magnitude is not bounded by
// construction (weights; activations behind a ReLU or no activation) therefore get their power of
// two at run time, from their largest magnitude or from a bound on it (split_pow2_scale): any finite
// fp32 value is then representable, and a non-finite one propagates as NaN / infinity as it would
// in fp32 arithmetic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evo {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kSplitLowScale = 2048.0f;           // 2^11: the residual term is stored times this
constexpr float kSplitLowUnscale = 1.0f / 2048.0f;  // factor of the second accumulator

// The power of two s that puts a tensor whose magnitudes are bounded by `bound` just below the top of
// fp16's range: s * bound in [2^14, 2^15).  s is limited to [2^-100, 2^64]: beyond 2^64 the values are
// below 2^-50 and simply sit lower in the format (they do not matter next to biases of any size that
// fp32 sums could hold them against); 2^-100 is reached only by bounds near the top of fp32's range.
__device__ __forceinline__ float split_pow2_scale(float bound) {
  const int E = (__float_as_int(bound) >> 23) & 0xff;  // biased exponent: bound in [2^(E-127), 2^(E-126))
  const int e = min(max(268 - E, 27), 191);            // biased exponent of s = 2^(14 - (E - 127))
  return __int_as_float(e << 23);
}
// 1 / s for a power of two s (exact).
__device__ __forceinline__ float pow2_reciprocal(float s) { return __int_as_float((254 << 23) - __float_as_int(s)); }

// Largest value over the 64 lanes of a wave, in every lane.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Two values -> the packed leading terms and the packed scaled residual terms.
__device__ __forceinline__ void split2_pair(float x0, float x1, uint32_t& lead, uint32_t& resid) {
  uint32_t hb = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x0, x1}, f16x2));
  asm volatile("" : "+v"(hb));  // one conversion: what is stored is what the residual is taken against
  const f16x2 h = __builtin_bit_cast(f16x2, hb);
  const f32x2 r = {(x0 - static_cast<float>(h[0])) * kSplitLowScale, (x1 - static_cast<float>(h[1])) * kSplitLowScale};
  lead = hb;
  resid = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, f16x2));
}

// Two values that are also at hand times 2^11 -> the packed leading terms and the packed scaled residual
// terms: the same numbers as split2_pair (x - h is exact, and so is its multiple), two instructions fewer.
__device__ __forceinline__ void split2_pair_scaled(float x0, float x1, float xs0, float xs1, uint32_t& lead,
                                                   uint32_t& resid) {
  uint32_t hb = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x0, x1}, f16x2));
  asm volatile("" : "+v"(hb));  // one conversion: what is stored is what the residual is taken against
  const f16x2 h = __builtin_bit_cast(f16x2, hb);
  const f32x2 r = {fmaf(static_cast<float>(h[0]), -kSplitLowScale, xs0),
                   fmaf(static_cast<float>(h[1]), -kSplitLowScale, xs1)};
  lead = hb;
  resid = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, f16x2));
}

// Eight values -> the two matrix operands (leading, residual).
__device__ __forceinline__ void split2_x8(const float x[8], f16x8& lead, f16x8& resid) {
  uint32_t l[4], r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2_pair(x[2 * i], x[2 * i + 1], l[i], r[i]);
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  lead = __builtin_bit_cast(f16x8, u32x4{l[0], l[1], l[2], l[3]});
  resid = __builtin_bit_cast(f16x8, u32x4{r[0], r[1], r[2], r[3]});
}

}  // namespace evo
