// fp32-accurate products on the 16-bit matrix instruction: two-term half-precision operand splits.
//
// A value x (already multiplied by a power of two s chosen per tensor so that its bound sits in
// [2^14, 2^15), well inside fp16's exponent range) is represented as x ~ h + m with h = fp16(x) and
// m = fp16(x - h): the residual is exact in fp32 and at most half an ulp of h, so it carries 11 more
// significand bits: |x - h - m| <= 2^-22 |x| as long as m is a normal number.  A product of two such
// values is accumulated in fp32 as h h' + h m' + m h' in ONE accumulator (three matrix instructions);
// every fp16 x fp16 product is exact in fp32 and the dropped m m' is below 2^-22 of the product.
//
// Three hardware facts shape the code.  (1) The matrix instruction takes half-precision subnormals as they
// are (measured: 2^-24 x 1024 = 2^-14), so m needs no factor of its own.  (An earlier form stored 2^11 m and
// kept h m' + m h' in a second accumulator that was added with the factor 2^-11 afterwards: one multiply-add
// per result, twice the accumulator registers, four more instructions per split pair.)  (2) v_cvt_pk_f16_f32,
// which the compiler picks for a pair of conversions, returns zero where the single conversion returns a
// subnormal.  The residual must be taken against the value that is actually stored, so the pair is converted
// once and the same register feeds both uses; and a residual below 2^-14 is dropped by the packed conversion
// (see split2_pair_true for what that costs and where the single conversions are used instead).  (3) The
// leading term overflows beyond 65504 / s.  Tensors whose magnitude is not bounded by construction (weights;
// activations behind a ReLU or no activation) therefore get their power of two at run time, from their largest
// magnitude or from a bound on it (split_pow2_scale): any finite fp32 value is then representable, and a
// non-finite one propagates as NaN / infinity as it would in fp32 arithmetic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evo {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

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

// Two values -> the packed leading terms and the packed residual terms x - h.  The packed conversion returns
// zero for a subnormal result, so a residual below 2^-14, which is that of a value below 2^-3, is dropped,
// and a value below 2^-14 altogether: the absolute error of a term is then at most 2^-14, against
// a tensor whose power of two puts its bound at 2^14 or above, i.e. 2^-28 of the bound (and 2^-22 of the
// value wherever the value is above 2^-3).
__device__ __forceinline__ void split2_pair_true(float x0, float x1, uint32_t& lead, uint32_t& resid) {
  uint32_t hb = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x0, x1}, f16x2));
  asm volatile("" : "+v"(hb));  // one conversion: what is stored is what the residual is taken against
  const f16x2 h = __builtin_bit_cast(f16x2, hb);
  const f32x2 r = {fmaf(static_cast<float>(h[0]), -1.0f, x0), fmaf(static_cast<float>(h[1]), -1.0f, x1)};
  lead = hb;
  resid = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, f16x2));
}
// The same with the residuals converted one by one, which keeps the subnormal ones (two instructions more per
// pair): for tensors that are split once and used for a whole launch (weights), where a value far below the
// tensor's bound must still keep (almost) its own 22 bits.
__device__ __forceinline__ void split2_pair_true_kept(float x0, float x1, uint32_t& lead, uint32_t& resid) {
  uint32_t hb = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x0, x1}, f16x2));
  asm volatile("" : "+v"(hb));
  const f16x2 h = __builtin_bit_cast(f16x2, hb);
  const float r0 = x0 - static_cast<float>(h[0]), r1 = x1 - static_cast<float>(h[1]);
  // (an empty statement between the two conversions keeps the compiler from pairing them)
  uint32_t lo = __builtin_bit_cast(uint16_t, static_cast<_Float16>(r0));
  asm volatile("" : "+v"(lo));
  const uint32_t hi = __builtin_bit_cast(uint16_t, static_cast<_Float16>(r1));
  lead = hb;
  resid = lo | (hi << 16);
}
// Eight values -> the two matrix operands (leading, residual itself); KEPT: subnormal residuals are kept.
template <bool KEPT>
__device__ __forceinline__ void split2_x8_true(const float x[8], f16x8& lead, f16x8& resid) {
  uint32_t l[4], r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (KEPT) split2_pair_true_kept(x[2 * i], x[2 * i + 1], l[i], r[i]);
    else split2_pair_true(x[2 * i], x[2 * i + 1], l[i], r[i]);
  }
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  lead = __builtin_bit_cast(f16x8, u32x4{l[0], l[1], l[2], l[3]});
  resid = __builtin_bit_cast(f16x8, u32x4{r[0], r[1], r[2], r[3]});
}

}  // namespace evo
