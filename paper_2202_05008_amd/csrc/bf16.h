// bfloat16 conversion helpers.  gfx950 rounds fp32 to bfloat16 (nearest even) in hardware
// (v_cvt_pk_bf16_f32, two values per instruction); the casts below compile to it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evo {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const bf16x2_t v = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ uint16_t to_bf16(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }

__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

}  // namespace evo
