// The fp32 MLP forward of one (member, tile of 64 samples) on the vector ALU, as a device function: the kernel of
// policy_mlp.hip runs it with the member's weights in memory, the one-launch generation of pgpe.hip with weights
// that it has just drawn into LDS.  Same instructions in the same order either way, so the two give the same bits.
#pragma once
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
  int pop;
};

// tanh without branches: 1 - 2 / (e^{2|x|} + 1) through the hardware's exp2 and reciprocal (absolute error about
// 1e-7, so 5e-7 relative from |x| = 0.25 on) and, below 0.25, the odd series up to x^9 (next term 9e-3 x^11: 2e-9
// relative); saturates to 1 for large |x| (e^{2|x|} = inf), propagates NaN.
__device__ __forceinline__ float tanh_fast_accurate(float x) {
  const float ax = fabsf(x);
  const float big = fmaf(-2.0f, __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(2.885390081777927f * ax) + 1.0f), 1.0f);
  const float x2 = ax * ax;
  float p = fmaf(x2, 62.0f / 2835.0f, -17.0f / 315.0f);
  p = fmaf(x2, p, 2.0f / 15.0f);
  p = fmaf(x2, p, -1.0f / 3.0f);
  p = fmaf(x2 * ax, p, ax);
  return copysignf(ax < 0.25f ? p : big, x);
}

__device__ __forceinline__ float activate(float x, int act) {
  if (act == EVO_ACT_TANH) return tanh_fast_accurate(x);
  if (act == EVO_ACT_RELU) return fmaxf(x, 0.f);
  return x;
}

// Sum over the 64 lanes of a wave in a fixed butterfly order (every lane gets the result).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// WPtr: pointer to the member's flat parameters (global memory: const float*; LDS: an address-space-3 pointer).
// lds: 2 * a.ldw * 64 floats.  Every thread of the 256 returns; nothing is left in flight.  With a loss, thread 0
// returns the tile's loss sum, which is also stored to a.partial when that is not null.
template <int LOSS, typename WPtr>
__device__ __forceinline__ float mlp_f32_body(const MlpArgs& a, WPtr theta, int member, int tile, float* lds) {
  constexpr int TB = kMlpTile;
  float* hin = lds;
  float* hout = lds + a.ldw * TB;
  const int tid = threadIdx.x;
  const int s = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b0 = tile * TB;
  const int b = b0 + s;
  const bool live = b < a.B;
  const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;
  const int D = a.sh.dims[0];
  // stage the observation tile transposed: hin[d][sample]
#pragma unroll 4
  for (int i = tid; i < D * TB; i += 256) {  // unrolled: the loads of four rounds are in flight together
    const int ss = i / D, d = i - ss * D;
    hin[d * TB + ss] = (b0 + ss < a.B) ? obs[static_cast<size_t>(b0 + ss) * D + d] : 0.f;
  }
  __syncthreads();
  int off = 0;
  for (int l = 0; l < a.sh.n_layers; ++l) {
    const int n_in = a.sh.dims[l], n_out = a.sh.dims[l + 1], act = a.sh.act[l];
    const WPtr W = theta + off;
    const WPtr bias = W + n_in * n_out;
    for (int o0 = wave * 4; o0 < n_out; o0 += 16) {
      float acc[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = (o0 + j < n_out) ? bias[o0 + j] : 0.f;
      if (o0 + 3 < n_out) {
        // unrolled so that the weight and activation reads of four k are issued before the first is waited for
        // (the sums still run in increasing k)
#pragma unroll 4
        for (int k = 0; k < n_in; ++k) {
          const float hk = hin[k * TB + s];
          const WPtr wr = W + k * n_out + o0;
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] = fmaf(hk, wr[j], acc[j]);
        }
      } else {
#pragma unroll 4
        for (int k = 0; k < n_in; ++k) {
          const float hk = hin[k * TB + s];
          const WPtr wr = W + k * n_out + o0;
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
    return 0.f;
  }
  if (wave != 0) return 0.f;
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
  if (s == 0 && a.partial) a.partial[static_cast<size_t>(member) * a.tiles + tile] = loss;
  return loss;
}

}  // namespace evo
