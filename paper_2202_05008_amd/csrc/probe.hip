// Rate probes: what this GPU actually delivers for the instruction kinds the roofline peaks are quoted
// for, so that a measured figure can be printed next to each published one (the benchmark calls them;
// no step of the neuroevolution path does).  Every wave runs `iters` rounds of eight independent
// instructions of one kind on registers only; the caller times the launch and divides.
#include "kernels.h"

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kProbeThreads = 256;
constexpr int kProbeBlocksPerCu = 8;  // 8 workgroups of 4 waves: 8 waves per SIMD when registers allow

// kind 0: fp32 fused multiply-add on the vector ALU (64 lanes x 2 flop per instruction)
__global__ __launch_bounds__(kProbeThreads) void probe_fma_f32(int iters, float* out) {
  float a[8];
  const float m = 1.0f + 1e-7f * threadIdx.x, c = 1e-9f * blockIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = 0.5f + 0.01f * i;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = fmaf(a[i], m, c);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += a[i];
  if (s == 12345.678f) out[0] = s;  // keeps the loop alive without a store in the common case
}

// kind 1: v_mfma_f32_16x16x32_f16 (16 x 16 x 32 x 2 flop per instruction)
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_f16(int iters, float* out) {
  halfx8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = static_cast<_Float16>(0.001f * (threadIdx.x + i)), b[i] = static_cast<_Float16>(0.5f);
  floatx4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
  if (s == 12345.678f) out[0] = s;
}

// kind 2: v_mfma_f32_32x32x16_bf16 (32 x 32 x 16 x 2 flop per instruction)
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_bf16(int iters, float* out) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = static_cast<__bf16>(0.001f * (threadIdx.x + i)), b[i] = static_cast<__bf16>(0.5f);
  floatx16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[i][k] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
  if (s == 12345.678f) out[0] = s;
}

// kind 3: v_mfma_f32_16x16x4_f32 (16 x 16 x 4 x 2 flop per instruction)
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_f32(int iters, float* out) {
  const float a = 0.001f * threadIdx.x, b = 0.5f;
  floatx4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
  if (s == 12345.678f) out[0] = s;
}

}  // namespace evo

using namespace evo;

extern "C" int evo_probe_rate(int32_t kind, int32_t iters, double* flop_out, float* out_dev, void* stream) {
  EVO_REQUIRE(flop_out != nullptr && out_dev != nullptr, EVO_ERR_ARG, "evo_probe_rate: null pointer");
  EVO_REQUIRE(kind >= 0 && kind <= 3, EVO_ERR_ARG, "evo_probe_rate: kind must be 0..3 (got %d)", kind);
  EVO_REQUIRE(iters >= 1 && iters <= (1 << 24), EVO_ERR_ARG, "evo_probe_rate: iters must be in [1, 2^24]");
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  EVO_REQUIRE(e == hipSuccess && cus > 0, EVO_ERR_HIP, "evo_probe_rate: no device: %s", hipGetErrorString(e));
  const dim3 grid(cus * kProbeBlocksPerCu), block(kProbeThreads);
  const double waves = static_cast<double>(grid.x) * (kProbeThreads / 64);
  static const double flop_per_instr[4] = {64.0 * 2, 16.0 * 16 * 32 * 2, 32.0 * 32 * 16 * 2, 16.0 * 16 * 4 * 2};
  hipStream_t s = as_stream(stream);
  switch (kind) {
    case 0: hipLaunchKernelGGL(probe_fma_f32, grid, block, 0, s, iters, out_dev); break;
    case 1: hipLaunchKernelGGL(probe_mfma_f16, grid, block, 0, s, iters, out_dev); break;
    case 2: hipLaunchKernelGGL(probe_mfma_bf16, grid, block, 0, s, iters, out_dev); break;
    default: hipLaunchKernelGGL(probe_mfma_f32, grid, block, 0, s, iters, out_dev); break;
  }
  *flop_out = waves * iters * 8.0 * flop_per_instr[kind];
  return check_launch("probe kernel");
}
