// Population-batched fp32 MLP forward: every member has its own weights, observations are
// shared or per member (Section 2, "Global Policy"; Section 4, "Exploring Novel Policy
// Architectures": get_actions passes a batch through one model whose parameters are data).
// The loss epilogue makes a supervised single-step task (Section 3, "Supervised Learning
// Tasks") one kernel: logits never leave the chip.
//
// Mapping: workgroup = (member, tile of 64 samples).  Lane = sample, so an activation
// h[k][sample] is one conflict-free LDS read; the four waves take different groups of four
// output neurons, whose weights W[k][o..o+3] are contiguous and wave-uniform (scalar loads).
#include "kernels.h"

namespace evo {

struct MlpArgs {
  MlpShape sh;
  const float* params;
  const float* obs;
  int64_t obs_stride;
  int B;
  float* out;
  const void* target;
  float* partial;
  int tiles;
  int ldw;  // LDS row capacity (max width)
};

__device__ __forceinline__ float activate(float x, int act) {
  if (act == EVO_ACT_TANH) return tanhf(x);
  if (act == EVO_ACT_RELU) return fmaxf(x, 0.f);
  return x;
}

// Sum over the 64 lanes of a wave in a fixed butterfly order (every lane gets the result).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <int LOSS>
__global__ __launch_bounds__(256) void mlp_f32_kernel(MlpArgs a) {
  extern __shared__ float lds[];
  constexpr int TB = kMlpTile;
  float* hin = lds;
  float* hout = lds + a.ldw * TB;
  const int tid = threadIdx.x;
  const int s = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int member = blockIdx.y;
  const int b0 = blockIdx.x * TB;
  const int b = b0 + s;
  const bool live = b < a.B;
  const float* theta = a.params + static_cast<size_t>(member) * a.sh.P;
  const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;
  const int D = a.sh.dims[0];
  // stage the observation tile transposed: hin[d][sample]
  for (int i = tid; i < D * TB; i += 256) {
    const int ss = i / D, d = i - ss * D;
    hin[d * TB + ss] = (b0 + ss < a.B) ? obs[static_cast<size_t>(b0 + ss) * D + d] : 0.f;
  }
  __syncthreads();
  int off = 0;
  for (int l = 0; l < a.sh.n_layers; ++l) {
    const int n_in = a.sh.dims[l], n_out = a.sh.dims[l + 1], act = a.sh.act[l];
    const float* W = theta + off;
    const float* bias = W + n_in * n_out;
    for (int o0 = wave * 4; o0 < n_out; o0 += 16) {
      float acc[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = (o0 + j < n_out) ? bias[o0 + j] : 0.f;
      if (o0 + 3 < n_out) {
        for (int k = 0; k < n_in; ++k) {
          const float hk = hin[k * TB + s];
          const float* wr = W + k * n_out + o0;
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] = fmaf(hk, wr[j], acc[j]);
        }
      } else {
        for (int k = 0; k < n_in; ++k) {
          const float hk = hin[k * TB + s];
          const float* wr = W + k * n_out + o0;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (o0 + j < n_out) acc[j] = fmaf(hk, wr[j], acc[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (o0 + j < n_out) hout[(o0 + j) * TB + s] = activate(acc[j], act);
    }
    __syncthreads();
    float* t = hin;
    hin = hout;
    hout = t;
    off += n_in * n_out + n_out;
  }
  // hin now holds the network output [A][sample]
  const int A = a.sh.dims[a.sh.n_layers];
  if (LOSS == LOSS_NONE) {
    float* dst = a.out + (static_cast<size_t>(member) * a.B + b0) * A;
    const int rows = min(TB, a.B - b0);
    for (int i = tid; i < rows * A; i += 256) {
      const int ss = i / A, o = i - ss * A;
      dst[i] = hin[o * TB + ss];
    }
    return;
  }
  if (wave != 0) return;
  float loss = 0.f;
  if (live) {
    if (LOSS == LOSS_CE) {
      const int y = min(max(static_cast<const int32_t*>(a.target)[b], 0), A - 1);  // labels outside [0, A) are clamped
      float mx = hin[s];
      for (int o = 1; o < A; ++o) mx = fmaxf(mx, hin[o * TB + s]);
      float se = 0.f;
      for (int o = 0; o < A; ++o) se += expf(hin[o * TB + s] - mx);
      loss = (mx + logf(se)) - hin[y * TB + s];
    } else {
      const float* tg = static_cast<const float*>(a.target) + (static_cast<size_t>(member) * a.B + b) * A;
      for (int o = 0; o < A; ++o) {
        const float d = hin[o * TB + s] - tg[o];
        loss = fmaf(d, d, loss);
      }
    }
  }
  loss = wave_sum(loss);
  if (s == 0) a.partial[static_cast<size_t>(member) * a.tiles + blockIdx.x] = loss;
}

int launch_mlp_f32(const MlpShape& sh, const float* params, const float* obs, int64_t obs_stride, int pop, int B,
                   float* out, int loss, const void* target, float* partial, hipStream_t s) {
  EVO_REQUIRE(sh.max_width <= 256, EVO_ERR_UNSUPPORTED, "fp32 MLP: layer widths above 256 are not supported (%d)",
              sh.max_width);
  MlpArgs a;
  a.sh = sh, a.params = params, a.obs = obs, a.obs_stride = obs_stride, a.B = B;
  a.out = out, a.target = target, a.partial = partial;
  a.tiles = (B + kMlpTile - 1) / kMlpTile;
  a.ldw = sh.max_width;
  const size_t shmem = sizeof(float) * 2 * a.ldw * kMlpTile;
  const dim3 grid(a.tiles, pop);
  auto launch = [&](auto kern) -> int {
    if (shmem > 64 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
      EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), shmem, s, a);
    return check_launch("mlp_f32_kernel");
  };
  if (loss == LOSS_NONE) return launch(mlp_f32_kernel<LOSS_NONE>);
  if (loss == LOSS_CE) return launch(mlp_f32_kernel<LOSS_CE>);
  return launch(mlp_f32_kernel<LOSS_MSE>);
}

// One wavefront per member: lanes read the partial sums coalesced (lane, lane + 64, ...) and the
// 64 lane totals are combined by a fixed butterfly, so the result does not depend on timing.
__global__ __launch_bounds__(64) void finalize_kernel(const float* __restrict__ partial, int pop, int n,
                                                      float scale, float* __restrict__ fitness) {
  const int m = blockIdx.x, lane = threadIdx.x;
  float acc = 0.f;
  for (int j = lane; j < n; j += 64) acc += partial[static_cast<size_t>(m) * n + j];
  acc = wave_sum(acc);
  if (lane == 0) fitness[m] = scale * acc;
}

int launch_finalize(const float* partial, int pop, int n, float scale, float* fitness, hipStream_t s) {
  hipLaunchKernelGGL(finalize_kernel, dim3(pop), dim3(64), 0, s, partial, pop, n, scale, fitness);
  return check_launch("finalize_kernel");
}

// ---- sphere --------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

// Workgroup (chunk, member) streams one contiguous piece of the member's row with 16-byte loads;
// x fastest, so consecutive workgroups read consecutive pieces of one row.  Per-thread order and
// the tree are fixed; the per-chunk sums are added in chunk order by finalize_kernel.
constexpr int kSphereChunk = 4096;  // parameters per workgroup (16 KB of fp32)

template <typename T>
__global__ __launch_bounds__(256) void sphere_kernel(const T* __restrict__ params,
                                                     const float* __restrict__ x_star, int P, int chunks,
                                                     float* __restrict__ partial) {
  __shared__ float red[4];
  const int tid = threadIdx.x;
  const T* row = params + static_cast<size_t>(blockIdx.y) * P;
  const int begin = blockIdx.x * kSphereChunk, end = min(P, begin + kSphereChunk);
  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  if (sizeof(T) == 4 && (P & 3) == 0) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4* r4 = reinterpret_cast<const f32x4*>(row);
    const float4* x4 = reinterpret_cast<const float4*>(x_star);
    for (int i = begin / 4 + tid; i < end / 4; i += 256) {
      const f32x4 p = __builtin_nontemporal_load(r4 + i);  // read once: keep it out of the caches
      const float4 x = x4[i];
      const float d0 = p.x - x.x, d1 = p.y - x.y, d2 = p.z - x.z, d3 = p.w - x.w;
      acc0 = fmaf(d0, d0, acc0);
      acc1 = fmaf(d1, d1, acc1);
      acc2 = fmaf(d2, d2, acc2);
      acc3 = fmaf(d3, d3, acc3);
    }
  } else {
    for (int i = begin + tid; i < end; i += 256) {
      float p;
      if (sizeof(T) == 4) p = reinterpret_cast<const float*>(row)[i];
      else p = bf16_to_f32(reinterpret_cast<const uint16_t*>(row)[i]);
      const float d = p - x_star[i];
      acc0 = fmaf(d, d, acc0);
    }
  }
  float acc = wave_sum((acc0 + acc1) + (acc2 + acc3));
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) partial[static_cast<size_t>(blockIdx.y) * chunks + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

int sphere_chunks(int P) { return (P + kSphereChunk - 1) / kSphereChunk; }

int launch_sphere(const void* params, int dtype, const float* x_star, int pop, int P, float* partial, float* fitness,
                  hipStream_t s) {
  const int chunks = sphere_chunks(P);
  const dim3 grid(chunks, pop);
  if (dtype == EVO_F32)
    hipLaunchKernelGGL(sphere_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(params), x_star, P,
                       chunks, partial);
  else
    hipLaunchKernelGGL(sphere_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(params), x_star,
                       P, chunks, partial);
  int rc = check_launch("sphere_kernel");
  if (rc) return rc;
  return launch_finalize(partial, pop, chunks, -1.0f, fitness, s);
}

}  // namespace evo
