// Population-batched fp32 MLP forward: every member has its own weights, observations are
// shared or per member (Section 2, "Global Policy"; Section 4, "Exploring Novel Policy
// Architectures": get_actions passes a batch through one model whose parameters are data).
// The loss epilogue makes a supervised single-step task (Section 3, "Supervised Learning
// Tasks") one kernel: logits never leave the chip.
//
// Mapping: workgroup = (member, tile of 64 samples).  Lane = sample, so an activation
// h[k][sample] is one conflict-free LDS read; the four waves take different groups of four
// output neurons, whose weights W[k][o..o+3] are contiguous and wave-uniform (scalar loads).
//
// Two kernels.  Networks whose layers are all narrow (every fan-in below 64: cfg1's 16-32-4) stay on the
// vector ALU (mlp_f32_kernel: they are bound by launch latency).  Any other network of widths up to 256 runs
// its layers as contractions on the matrix cores (mlp_f32_mfma_kernel): fp32 operands as two-term scaled fp16
// splits (split16.h), three v_mfma_f32_16x16x32_f16 per product, fp32 accumulation, results within a few
// 1e-7 of fp32 arithmetic.
#include "kernels.h"
#include "mlp_f32_body.h"
#include "split16.h"

namespace evo {

template <int LOSS>
__global__ __launch_bounds__(256) void mlp_f32_kernel(MlpArgs a) {
  extern __shared__ float lds[];
  mlp_f32_body<LOSS>(a, a.params + static_cast<size_t>(blockIdx.y) * a.sh.P, blockIdx.y, blockIdx.x, lds);
}

// ---- the matrix-core form ------------------------------------------------------------------------------
// Workgroup = (member, tile of 64 samples), eight waves (two per SIMD).  A layer is computed
// transposed: rows of a 16 x 16 tile are neurons (A operand: the member's weights W[k][neuron], fetched one
// tile ahead of their use and split once per neuron tile), columns are samples (B operand: the layer's input,
// kept in LDS as two fp16 terms [term][sample][k], one 16-byte read per term and 32 k).  A lane then ends up
// with four consecutive neurons of one sample: bias, activation, and one 8-byte LDS store per term hand them
// to the next layer.  Wave w takes neuron tiles w, w + 8, ...; its outputs wait in registers until every wave
// has finished reading the layer's input, which they then overwrite.
// Scales (powers of two, so that every finite fp32 value fits fp16's range): the weights of a neuron tile from
// their largest magnitude; the activations of a SAMPLE from the largest magnitude among that sample's outputs
// of the layer (in-lane maxima, two lane exchanges, one LDS word per wave and sample).  The factor of a
// pre-activation, 1 / (sample scale x tile scale), rides in the multiply-add that adds the bias.
typedef float floatx4m __attribute__((ext_vector_type(4)));
constexpr int kMfmaMaxWidth = 256;             // fan-in and fan-out of a layer
constexpr int kMfmaKSteps = kMfmaMaxWidth / 32;
constexpr int kMfmaWaves = 8;
constexpr int kMfmaSlots = kMfmaMaxWidth / 16 / kMfmaWaves;  // neuron tiles per wave

template <int LOSS>
__global__ __launch_bounds__(64 * kMfmaWaves, 2) void mlp_f32_mfma_kernel(MlpArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  constexpr int TB = kMlpTile;
  static_assert(TB == 64, "four column tiles of 16 samples");
  const int kRowB = (a.ldw + 8) * 2;       // bytes of one sample's row of one term (a.ldw: widest padded fan-in)
  const int kTermB = TB * kRowB;
  unsigned char* at = lds_raw;                                    // [2][64][ldw + 8] fp16
  float* smax = reinterpret_cast<float*>(lds_raw + 2 * kTermB);   // [8][64] per wave: largest |output| of a sample
  float* us_s = smax + kMfmaWaves * TB;                                    // [64] 1 / scale of the staged observations
  float* fin = reinterpret_cast<float*>(lds_raw);                 // [A][64] network output (after the last layer)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, q = lane >> 4;
  // Workgroup -> (member, tile): consecutive workgroup numbers go to the eight dies in turn, each with a cache
  // of its own, so a member's tiles, which read the same weights, take numbers that are 8 apart.
  const int die = blockIdx.x & 7, turn = blockIdx.x >> 3;
  const int member = 8 * (turn / a.tiles) + die, tile = turn % a.tiles, b0 = tile * TB;
  if (member >= a.pop) return;
  const float* theta = a.params + static_cast<size_t>(member) * a.sh.P;
  const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;

  // ---- observations -> two fp16 terms per value, scaled per sample (eight threads per sample) --------------
  {
    const int D = a.sh.dims[0], KP = (D + 31) & ~31;
    const int smp = tid >> 3, part = tid & 7;
    const bool live = b0 + smp < a.B;
    const float* row = obs + static_cast<size_t>(b0 + smp) * D;
    float sc;
    if ((D & 3) == 0 && (reinterpret_cast<uintptr_t>(obs) & 15u) == 0) {  // then every row starts on 16 bytes
      // every 16-byte load of the thread's share of the row is in flight at once: one trip to memory
      float4 v[kMfmaMaxWidth / 32];
      float m = 0.f;
#pragma unroll
      for (int c = 0; c < kMfmaMaxWidth / 32; ++c) {
        const int d = 4 * (part + 8 * c);
        v[c] = (live && d < D) ? *reinterpret_cast<const float4*>(row + d) : make_float4(0.f, 0.f, 0.f, 0.f);
        m = fmaxf(fmaxf(m, fmaxf(fabsf(v[c].x), fabsf(v[c].y))), fmaxf(fabsf(v[c].z), fabsf(v[c].w)));
      }
      m = fmaxf(m, __shfl_xor(m, 1, 64));
      m = fmaxf(m, __shfl_xor(m, 2, 64));
      m = fmaxf(m, __shfl_xor(m, 4, 64));
      sc = split_pow2_scale(m);
#pragma unroll
      for (int c = 0; c < kMfmaMaxWidth / 32; ++c) {
        const int d = 4 * (part + 8 * c);
        if (d < KP) {
          uint2 lead, resid;
          split2_pair_true(sc * v[c].x, sc * v[c].y, lead.x, resid.x);
          split2_pair_true(sc * v[c].z, sc * v[c].w, lead.y, resid.y);
          *reinterpret_cast<uint2*>(at + smp * kRowB + d * 2) = lead;
          *reinterpret_cast<uint2*>(at + kTermB + smp * kRowB + d * 2) = resid;
        }
      }
    } else {
      float m = 0.f;
      for (int d = part; d < D; d += 8) m = fmaxf(m, live ? fabsf(row[d]) : 0.f);
      m = fmaxf(m, __shfl_xor(m, 1, 64));
      m = fmaxf(m, __shfl_xor(m, 2, 64));
      m = fmaxf(m, __shfl_xor(m, 4, 64));
      sc = split_pow2_scale(m);
      for (int d = 2 * part; d < KP; d += 16) {
        const float x0 = (live && d < D) ? sc * row[d] : 0.f, x1 = (live && d + 1 < D) ? sc * row[d + 1] : 0.f;
        uint32_t lead, resid;
        split2_pair_true(x0, x1, lead, resid);
        *reinterpret_cast<uint32_t*>(at + smp * kRowB + d * 2) = lead;
        *reinterpret_cast<uint32_t*>(at + kTermB + smp * kRowB + d * 2) = resid;
      }
    }
    if (part == 0) us_s[smp] = pow2_reciprocal(sc);
  }
  __syncthreads();
  float u_s[4];  // 1 / scale of the stored input of sample 16 ct + j
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) u_s[ct] = us_s[16 * ct + j];

  // A neuron tile's weights as A operands, A[row j][k = 32 s + 8 q + e] = W[k][16 nt + j], and its four biases
  // per lane, are fetched one tile ahead: all 64 loads of the next tile are in flight while the matrix
  // instructions of this one run.
  float raw[kMfmaKSteps][8], bias4[4];
  const int n_layers = a.sh.n_layers;
  auto tiles_of = [&](int l) {  // neuron tiles of layer l: its outputs fill the next fan-in up to a multiple of 32
    const int N = a.sh.dims[l + 1];
    return l == n_layers - 1 ? (N + 15) >> 4 : ((N + 31) & ~31) >> 4;
  };
  // Fetches this wave's first tile at or after (layer l, slot).  Loads go to clamped addresses, so that none is
  // predicated or waited for here; what lies beyond the layer's fan-in or fan-out is zeroed where the tile is used.
  auto fetch_from = [&](int l, int slot, const float* W) {
    while (l < n_layers && !(slot < kMfmaSlots && wave + kMfmaWaves * slot < tiles_of(l))) {
      W += a.sh.dims[l] * a.sh.dims[l + 1] + a.sh.dims[l + 1];
      ++l, slot = 0;
    }
    if (l >= n_layers) return;
    const int K = a.sh.dims[l], N = a.sh.dims[l + 1], nt = wave + kMfmaWaves * slot;
    const int KS = (K + 31) >> 5;
    // address = a wave-uniform row pointer + an unsigned per-lane offset (no per-load vector arithmetic); only
    // a ragged last step clamps its rows per lane
    const unsigned lane_off = 4u * static_cast<unsigned>(8 * q * N + min(16 * nt + j, N - 1));  // bytes
#pragma unroll
    for (int st = 0; st < kMfmaKSteps; ++st) {
      if (st < KS) {
        if (32 * st + 32 <= K) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            raw[st][e] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(W + (32 * st + e) * N) + lane_off);
        } else {
          const unsigned col = static_cast<unsigned>(min(16 * nt + j, N - 1));
#pragma unroll
          for (int e = 0; e < 8; ++e) raw[st][e] = W[static_cast<unsigned>(min(32 * st + 8 * q + e, K - 1) * N) + col];
        }
      }
    }
    const float* bias = W + K * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int o = 16 * nt + 4 * q + i;
      bias4[i] = bias[min(o, N - 1)];
    }
  };
  fetch_from(0, 0, theta);

  int off = 0;
  for (int l = 0; l < n_layers; ++l) {
    const int K = a.sh.dims[l], N = a.sh.dims[l + 1], act = a.sh.act[l];
    const bool last = l == n_layers - 1;
    const int KS = (K + 31) >> 5;
    const int NT = tiles_of(l);
    const float* W = theta + off;
    float held[kMfmaSlots][4][4];  // [slot][sample tile][neuron 4 q + i]: this wave's outputs of the layer
    float m_s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int slot = 0; slot < kMfmaSlots; ++slot) {
      const int nt = wave + kMfmaWaves * slot;
      if (nt >= NT) continue;
      // ---- zeros beyond a ragged fan-in or fan-out, scale from the tile's largest magnitude, split ----
      if ((K & 31) != 0 || 16 * nt + 16 > N) {
        const bool ok = 16 * nt + j < N;
#pragma unroll
        for (int st = 0; st < kMfmaKSteps; ++st) {
          if (st < KS) {
#pragma unroll
            for (int e = 0; e < 8; ++e) raw[st][e] = (ok && 32 * st + 8 * q + e < K) ? raw[st][e] : 0.f;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) bias4[i] = 16 * nt + 4 * q + i < N ? bias4[i] : 0.f;
      }
      float w_max = 0.f;
#pragma unroll
      for (int st = 0; st < kMfmaKSteps; ++st) {
        if (st < KS) {
#pragma unroll
          for (int e = 0; e < 8; ++e) w_max = fmaxf(w_max, fabsf(raw[st][e]));
        }
      }
      const float s_w = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(wave_max(w_max)))));
      const float u_w = pow2_reciprocal(s_w);
      f16x8 wa[2][kMfmaKSteps];
#pragma unroll
      for (int st = 0; st < kMfmaKSteps; ++st) {
        if (st < KS) {
#pragma unroll
          for (int e = 0; e < 8; ++e) raw[st][e] *= s_w;
          split2_x8_true<false>(raw[st], wa[0][st], wa[1][st]);
        }
      }
      float b4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) b4[i] = bias4[i];
      // ---- this wave's next tile: the layer's second one, else the first of a later layer ----
      fetch_from(l, slot + 1, W);
      // ---- four sample tiles ----
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        floatx4m acc = {0.f, 0.f, 0.f, 0.f};  // all three partial products (residual terms unscaled)
        const unsigned char* src = at + (16 * ct + j) * kRowB + 16 * q;
#pragma unroll
        for (int st = 0; st < kMfmaKSteps; ++st) {
          if (st < KS) {
            const f16x8 x0 = *reinterpret_cast<const f16x8*>(src + 64 * st);
            const f16x8 x1 = *reinterpret_cast<const f16x8*>(src + kTermB + 64 * st);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0][st], x1, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[1][st], x0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0][st], x0, acc, 0, 0, 0);
          }
        }
        const float u = u_s[ct] * u_w;
#pragma unroll
        for (int i = 0; i < 4; ++i) held[slot][ct][i] = fmaf(acc[i], u, b4[i]);
      }
      // the activation of the tile's sixteen values per lane, switched once and not per value
      auto apply = [&](auto f) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float v = f(held[slot][ct][i]);
            held[slot][ct][i] = v;
            m_s[ct] = fmaxf(m_s[ct], fabsf(v));
          }
      };
      if (act == EVO_ACT_TANH) apply([](float x) { return tanh_fast_accurate(x); });
      else if (act == EVO_ACT_RELU) apply([](float x) { return fmaxf(x, 0.f); });
      else apply([](float x) { return x; });
    }
    if (last) {
      __syncthreads();  // every wave has read the layer's input: the buffer takes the network's output
#pragma unroll
      for (int slot = 0; slot < kMfmaSlots; ++slot) {
        const int nt = wave + kMfmaWaves * slot;
        if (nt >= NT) continue;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int o = 16 * nt + 4 * q + i;
            if (o < N) fin[o * TB + 16 * ct + j] = held[slot][ct][i];
          }
      }
      __syncthreads();
      break;
    }
    // ---- per-sample scale of this layer's outputs: the largest magnitude over all neurons ----
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      float m = m_s[ct];
      m = fmaxf(m, __shfl_xor(m, 16, 64));
      m = fmaxf(m, __shfl_xor(m, 32, 64));
      if (q == 0) smax[wave * TB + 16 * ct + j] = m;
    }
    __syncthreads();  // every wave has read the layer's input, and the maxima are out
    float s_new[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      const int smp = 16 * ct + j;
      float m = smax[smp];
#pragma unroll
      for (int w = 1; w < kMfmaWaves; ++w) m = fmaxf(m, smax[w * TB + smp]);
      s_new[ct] = split_pow2_scale(m);
      u_s[ct] = pow2_reciprocal(s_new[ct]);
    }
#pragma unroll
    for (int slot = 0; slot < kMfmaSlots; ++slot) {
      const int nt = wave + kMfmaWaves * slot;
      if (nt >= NT) continue;
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        uint2 lead, resid;
        split2_pair_true(s_new[ct] * held[slot][ct][0], s_new[ct] * held[slot][ct][1], lead.x, resid.x);
        split2_pair_true(s_new[ct] * held[slot][ct][2], s_new[ct] * held[slot][ct][3], lead.y, resid.y);
        unsigned char* dst = at + (16 * ct + j) * kRowB + (16 * nt + 4 * q) * 2;
        *reinterpret_cast<uint2*>(dst) = lead;
        *reinterpret_cast<uint2*>(dst + kTermB) = resid;
      }
    }
    __syncthreads();
    off += K * N + N;
  }

  // ---- the network output [A][sample] -> memory, or its loss (as in mlp_f32_kernel) -----------------------
  const int A = a.sh.dims[n_layers];
  const int s = tid & 63, b = b0 + s;
  if (LOSS == LOSS_NONE) {
    float* dst = a.out + (static_cast<size_t>(member) * a.B + b0) * A;
    const int rows = min(TB, a.B - b0);
    for (int i = tid; i < rows * A; i += 64 * kMfmaWaves) {
      const int ss = i / A, o = i - ss * A;
      dst[i] = fin[o * TB + ss];
    }
    return;
  }
  if (wave != 0) return;
  float loss = 0.f;
  if (b < a.B) {
    if (LOSS == LOSS_CE) {
      const int y = min(max(static_cast<const int32_t*>(a.target)[b], 0), A - 1);  // labels outside [0, A) are clamped
      float mx = fin[s];
      for (int o = 1; o < A; ++o) mx = fmaxf(mx, fin[o * TB + s]);
      float se = 0.f;
      for (int o = 0; o < A; ++o) se += expf(fin[o * TB + s] - mx);
      loss = (mx + logf(se)) - fin[y * TB + s];
    } else {
      const float* tg = static_cast<const float*>(a.target) + (static_cast<size_t>(member) * a.B + b) * A;
      for (int o = 0; o < A; ++o) {
        const float d = fin[o * TB + s] - tg[o];
        loss = fmaf(d, d, loss);
      }
    }
  }
  loss = wave_sum(loss);
  if (s == 0) a.partial[static_cast<size_t>(member) * a.tiles + tile] = loss;
}

// The matrix-core kernel takes networks of widths up to 256 with at least one fan-in of 64 or more.
static bool mfma_shape(const MlpShape& sh) {
  if (sh.max_width > kMfmaMaxWidth) return false;
  for (int l = 0; l < sh.n_layers; ++l)
    if (sh.dims[l] >= 64) return true;
  return false;
}

int launch_mlp_f32(const MlpShape& sh, const float* params, const float* obs, int64_t obs_stride, int pop, int B,
                   float* out, int loss, const void* target, float* partial, hipStream_t s) {
  EVO_REQUIRE(sh.max_width <= 256, EVO_ERR_UNSUPPORTED, "fp32 MLP: layer widths above 256 are not supported (%d)",
              sh.max_width);
  MlpArgs a;
  a.sh = sh, a.params = params, a.obs = obs, a.obs_stride = obs_stride, a.B = B;
  a.out = out, a.target = target, a.partial = partial;
  a.tiles = (B + kMlpTile - 1) / kMlpTile;
  a.pop = pop;
  const dim3 grid(a.tiles, pop);
  if (mfma_shape(sh)) {
    int kp = 32;      // widest fan-in, padded to the matrix instruction's 32
    for (int l = 0; l < sh.n_layers; ++l) kp = max(kp, (sh.dims[l] + 31) & ~31);
    a.ldw = kp;
    const size_t lds = static_cast<size_t>(2) * kMlpTile * (kp + 8) * 2 + (kMfmaWaves + 1) * kMlpTile * sizeof(float);
    auto launch_mfma = [&](auto kern) -> int {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
      if (e != hipSuccess) (void)hipGetLastError();
      EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
      hipLaunchKernelGGL(kern, dim3(8 * ((pop + 7) / 8) * a.tiles), dim3(64 * kMfmaWaves), lds, s, a);
      return check_launch("mlp_f32_mfma_kernel");
    };
    if (loss == LOSS_NONE) return launch_mfma(mlp_f32_mfma_kernel<LOSS_NONE>);
    if (loss == LOSS_CE) return launch_mfma(mlp_f32_mfma_kernel<LOSS_CE>);
    return launch_mfma(mlp_f32_mfma_kernel<LOSS_MSE>);
  }
  a.ldw = sh.max_width;
  const size_t shmem = sizeof(float) * 2 * a.ldw * kMlpTile;
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
