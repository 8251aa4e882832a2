// Device-side Philox4x32-10 and the word -> standard normal transform used by ask and tell.
//
// Generator: Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3"
// (SC'11).  The EvoJAX paper only speaks of seeding by keys (Section 4); the counter
// layout (i >> 2, pair, generation, tag) with key = the two halves of the 64-bit seed lets
// ask and tell regenerate any perturbation instead of storing it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evo {

struct u32x4 {
  uint32_t x, y, z, w;
};

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32x32 -> 64 bit multiply per lane pair (v_mad_u64_u32 gives both halves)
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    // three-input xor in one instruction (v_bitop3_b32, truth table 0x96 = odd parity)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p0 >> 32), c3, k1, 0x96);
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return u32x4{c0, c1, c2, c3};
}

// (2 (x >> 9) + 1) 2^-24: an odd multiple of 2^-24 in (0,1).  Built without an integer
// conversion: the 23 bits become the fraction of a float f in [1, 2), and f - (1 - 2^-24) is that
// value exactly (the difference is an odd multiple of 2^-24 below 1, hence representable).
__device__ __forceinline__ float unit_open(uint32_t x) {
  return __uint_as_float((x >> 9) | 0x3F800000u) - 0.999999940395355224609375f;
}

// Box-Muller on two words: za = r cos(2 pi ub), zb = r sin(2 pi ub), r = sqrt(-2 ln ua).
// The hardware transcendentals fit the inputs exactly: v_sin_f32 / v_cos_f32 take the angle in
// revolutions, so ub goes in unrounded, and v_log_f32 is a base-2 logarithm, so
// -2 ln ua = -(2 ln 2) log2 ua.  Measured over all 2^23 possible inputs against fp64: sine and
// cosine within 1.3e-7 absolute, r within 1.4e-7 relative.
__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& za, float& zb) {
  const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(unit_open(xa)));
  const float ub = unit_open(xb);
  za = r * __builtin_amdgcn_cosf(ub);
  zb = r * __builtin_amdgcn_sinf(ub);
}

// Four standard normals of counter (j, pair, gen, tag).
__device__ __forceinline__ void philox_normal4(uint32_t j, uint32_t pair, uint32_t gen, uint32_t tag, uint32_t k0,
                                               uint32_t k1, float z[4]) {
  const u32x4 w = philox4x32_10(j, pair, gen, tag, k0, k1);
  box_muller(w.x, w.y, z[0], z[1]);
  box_muller(w.z, w.w, z[2], z[3]);
}

}  // namespace evo
