// PGPE ask / tell for gfx950 (Section 4, "Devising New Algorithms": ask generates a
// population of parameters, tell reports the evaluation results back for the state update;
// PGPE is the algorithm named in Section 5; Section 2, "Modern ML Optimizers": the gradient
// estimate is handed to an Adam-class optimizer).
//
// Design: the perturbations are never stored.  ask streams mu and sigma once and writes the
// population; tell regenerates every normal from the counter-based generator, reduces the
// rank-weighted sums in registers / LDS in a fixed order and applies the optimizer in the
// same kernel, so mu, sigma and the moments are read and written exactly once.
#include "kernels.h"
#include "mlp_f32_body.h"
#include "philox.h"
#include "bf16.h"

#include <math.h>
#include <string.h>
#include <new>

struct pgpe_state {
  pgpe_config cfg;
  float* mu;
  float* sigma;
  float* m;
  float* v;
  float* aux;
  void* work;
  uint32_t t;
  bool device_t;  // the generation index also lives on the device and the kernels read it there
  bool pending;
  uint64_t seed;
  int32_t pop;
  bool tickets_ready;  // the two counters of the one-launch generation have been cleared
};

namespace evo {

// ---- workspace layout ------------------------------------------------------------------
constexpr int kNormBlocks = 256;  // partial sums of a squared norm over P (ClipUp)

struct Workspace {
  float* shaped;   // [pop_max] utilities c_m
  uint32_t* rank;  // [pop_max]
  float* norm;     // [2][kNormBlocks] partial sums of |g|^2 and |vel|^2
  uint32_t* gen;   // generation index t on the device (used once pgpe_device_generation has been called)
};

static inline size_t ws_arrays_bytes(int pop_max) {
  return ((static_cast<size_t>(pop_max) * 2 + 2 * kNormBlocks) * 4 + 255) & ~size_t(255);
}
constexpr int kSmallSumWords = 2 * 4096;  // the two arrays of loss sums of the one-launch generation
static inline size_t ws_bytes(int pop_max) { return ws_arrays_bytes(pop_max) + 256 + 4 * kSmallSumWords; }

static inline Workspace ws_carve(void* base, int pop_max) {
  Workspace w;
  w.shaped = static_cast<float*>(base);
  w.rank = reinterpret_cast<uint32_t*>(w.shaped + pop_max);
  w.norm = reinterpret_cast<float*>(w.rank + pop_max);
  w.gen = reinterpret_cast<uint32_t*>(static_cast<char*>(base) + ws_arrays_bytes(pop_max));
  return w;
}

// ---- ask -------------------------------------------------------------------------------
__device__ __forceinline__ void store_row4(float* row, int col, int P, const float v[4], bool vec) {
  if (vec) {
    // streaming store: the population is written once and read by a later kernel
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4*>(row + col));
  } else if ((P & 1) == 0 && col + 3 < P) {
    // even P: rows are 8-byte aligned, two 8-byte streaming stores
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store(f32x2{v[0], v[1]}, reinterpret_cast<f32x2*>(row + col));
    __builtin_nontemporal_store(f32x2{v[2], v[3]}, reinterpret_cast<f32x2*>(row + col + 2));
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (col + i < P) row[col + i] = v[i];
  }
}

__device__ __forceinline__ void store_row4(uint16_t* row, int col, int P, const float v[4], bool vec) {
  if (vec) {
    uint2 pk;
    pk.x = pack_bf16x2(v[0], v[1]);
    pk.y = pack_bf16x2(v[2], v[3]);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store(u32x2{pk.x, pk.y}, reinterpret_cast<u32x2*>(row + col));
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (col + i < P) row[col + i] = to_bf16(v[i]);
  }
}

// One thread owns four consecutive parameters (one Philox counter) and walks over a chunk
// of pairs; mu and sigma are loaded once per thread, the two mirrored rows share one draw.
template <typename OutT>
__global__ __launch_bounds__(256) void ask_kernel(const float* __restrict__ mu, const float* __restrict__ sigma,
                                                  OutT* __restrict__ params, int P, int nquads, int N,
                                                  int pairs_per_block, uint32_t gen_host,
                                                  const uint32_t* __restrict__ gen_dev, uint32_t key0, uint32_t key1) {
  const uint32_t gen = gen_dev ? *gen_dev : gen_host;  // uniform: the device copy when the state keeps one
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= nquads) return;
  const int col = q * 4;
  const bool vec = (P & 3) == 0;  // rows are 16-byte (fp32) / 8-byte (bf16) aligned only then
  float mu4[4], sg4[4];
  if (col + 3 < P) {
    const float4 a = *reinterpret_cast<const float4*>(mu + col);
    const float4 b = *reinterpret_cast<const float4*>(sigma + col);
    mu4[0] = a.x, mu4[1] = a.y, mu4[2] = a.z, mu4[3] = a.w;
    sg4[0] = b.x, sg4[1] = b.y, sg4[2] = b.z, sg4[3] = b.w;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mu4[i] = col + i < P ? mu[col + i] : 0.f;
      sg4[i] = col + i < P ? sigma[col + i] : 0.f;
    }
  }
  const int k_begin = blockIdx.y * pairs_per_block;
  const int k_end = min(N, k_begin + pairs_per_block);
  for (int k = k_begin; k < k_end; ++k) {
    float z[4], plus[4], minus[4];
    philox_normal4(static_cast<uint32_t>(q), static_cast<uint32_t>(k), gen, EVO_TAG_NOISE, key0, key1, z);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // both members from the exact product: each is rounded once, so they mirror about mu
      plus[i] = fmaf(sg4[i], z[i], mu4[i]);
      minus[i] = fmaf(-sg4[i], z[i], mu4[i]);
    }
    OutT* row = params + static_cast<size_t>(2 * k) * P;
    store_row4(row, col, P, plus, vec);
    store_row4(row + P, col, P, minus, vec);
  }
}

// bfloat16 population with P a multiple of 8: one thread owns eight consecutive parameters (two
// Philox counters) of one pair, so that each row takes one 16-byte streaming store per thread.
__global__ __launch_bounds__(256) void ask_bf16x8_kernel(const float* __restrict__ mu, const float* __restrict__ sigma,
                                                         uint16_t* __restrict__ params, int P, int noct,
                                                         uint32_t gen_host, const uint32_t* __restrict__ gen_dev,
                                                         uint32_t key0, uint32_t key1) {
  const uint32_t gen = gen_dev ? *gen_dev : gen_host;
  const int o = blockIdx.x * 256 + threadIdx.x;
  if (o >= noct) return;
  const int col = o * 8, k = blockIdx.y;
  const float4 ma = *reinterpret_cast<const float4*>(mu + col), mb = *reinterpret_cast<const float4*>(mu + col + 4);
  const float4 sa = *reinterpret_cast<const float4*>(sigma + col), sb = *reinterpret_cast<const float4*>(sigma + col + 4);
  const float mu8[8] = {ma.x, ma.y, ma.z, ma.w, mb.x, mb.y, mb.z, mb.w};
  const float sg8[8] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
  float z[8];
  philox_normal4(static_cast<uint32_t>(2 * o), static_cast<uint32_t>(k), gen, EVO_TAG_NOISE, key0, key1, z);
  philox_normal4(static_cast<uint32_t>(2 * o + 1), static_cast<uint32_t>(k), gen, EVO_TAG_NOISE, key0, key1, z + 4);
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 plus, minus;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    plus[i] = pack_bf16x2(fmaf(sg8[2 * i], z[2 * i], mu8[2 * i]), fmaf(sg8[2 * i + 1], z[2 * i + 1], mu8[2 * i + 1]));
    minus[i] = pack_bf16x2(fmaf(-sg8[2 * i], z[2 * i], mu8[2 * i]), fmaf(-sg8[2 * i + 1], z[2 * i + 1], mu8[2 * i + 1]));
  }
  uint16_t* row = params + static_cast<size_t>(2 * k) * P + col;
  __builtin_nontemporal_store(plus, reinterpret_cast<u32x4*>(row));
  __builtin_nontemporal_store(minus, reinterpret_cast<u32x4*>(row + P));
}

// ---- ask fused with the sphere fitness: the population is never written --------------------------
// Thread = kFusedQuads parameter quads x kFusedPairs pairs: mu, sigma and x_star are loaded once
// per quad, each draw serves both members of its pair, and theta is formed exactly as ask_kernel
// stores it (one fused multiply-add, rounded once) before x_star is subtracted.  A workgroup
// leaves one partial sum per member in part[member][blockIdx.x]; sphere_finish_kernel adds a
// member's partial sums in a fixed order.
constexpr int kFusedQuads = 4;
constexpr int kFusedPairs = 4;

__global__ __launch_bounds__(256) void ask_sphere_kernel(const float* __restrict__ mu, const float* __restrict__ sigma,
                                                         const float* __restrict__ x_star, float* __restrict__ part,
                                                         int P, int nquads, int N, int xblocks, uint32_t gen_host,
                                                         const uint32_t* __restrict__ gen_dev, uint32_t key0,
                                                         uint32_t key1) {
  const uint32_t gen = gen_dev ? *gen_dev : gen_host;
  __shared__ float red[4][2 * kFusedPairs];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k0 = blockIdx.y * kFusedPairs;
  float acc[kFusedPairs][2];
#pragma unroll
  for (int ki = 0; ki < kFusedPairs; ++ki) acc[ki][0] = acc[ki][1] = 0.f;
  for (int qi = 0; qi < kFusedQuads; ++qi) {
    const int q = (blockIdx.x * kFusedQuads + qi) * 256 + tid;
    if (q >= nquads) break;
    const int col = q * 4;
    float mu4[4], sg4[4], xs4[4];
    if (col + 3 < P) {
      const float4 a = *reinterpret_cast<const float4*>(mu + col);
      const float4 b = *reinterpret_cast<const float4*>(sigma + col);
      const float4 c = *reinterpret_cast<const float4*>(x_star + col);
      mu4[0] = a.x, mu4[1] = a.y, mu4[2] = a.z, mu4[3] = a.w;
      sg4[0] = b.x, sg4[1] = b.y, sg4[2] = b.z, sg4[3] = b.w;
      xs4[0] = c.x, xs4[1] = c.y, xs4[2] = c.z, xs4[3] = c.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {  // columns beyond P contribute (0 - 0)^2
        mu4[i] = col + i < P ? mu[col + i] : 0.f;
        sg4[i] = col + i < P ? sigma[col + i] : 0.f;
        xs4[i] = col + i < P ? x_star[col + i] : 0.f;
      }
    }
#pragma unroll
    for (int ki = 0; ki < kFusedPairs; ++ki) {
      if (k0 + ki >= N) break;  // uniform over the workgroup
      float z[4];
      philox_normal4(static_cast<uint32_t>(q), static_cast<uint32_t>(k0 + ki), gen, EVO_TAG_NOISE, key0, key1, z);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float dp = fmaf(sg4[i], z[i], mu4[i]) - xs4[i];
        const float dm = fmaf(-sg4[i], z[i], mu4[i]) - xs4[i];
        acc[ki][0] = fmaf(dp, dp, acc[ki][0]);
        acc[ki][1] = fmaf(dm, dm, acc[ki][1]);
      }
    }
  }
#pragma unroll
  for (int ki = 0; ki < kFusedPairs; ++ki)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      float v = acc[ki][s];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      if (lane == 0) red[wave][2 * ki + s] = v;
    }
  __syncthreads();
  if (tid < 2 * kFusedPairs && k0 + (tid >> 1) < N) {
    const float total = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
    part[static_cast<size_t>(2 * k0 + tid) * xblocks + blockIdx.x] = total;
  }
}

// fitness[m] = -(sum of the member's xblocks partial sums): one wavefront per member, lane l adds
// partial sums l, l + 64, ... in order, then a fixed butterfly over the lanes.
__global__ __launch_bounds__(256) void sphere_finish_kernel(const float* __restrict__ part, int xblocks, int pop,
                                                            float* __restrict__ fitness) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= pop) return;
  const float* row = part + static_cast<size_t>(m) * xblocks;
  float v = 0.f;
  for (int i = lane; i < xblocks; i += 64) v += row[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  if (lane == 0) fitness[m] = -v;
}

static inline int fused_xblocks(int P) { return ((P + 3) / 4 + 256 * kFusedQuads - 1) / (256 * kFusedQuads); }

// ---- centered ranks and pair weights ------------------------------------------------------
// fp32 bits -> u32 that orders like the float: -0 counts as +0, NaN sorts lowest.
__device__ __forceinline__ uint32_t orderable(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0u;
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Centered ranks by counting: the rank of member m is the number of 64-bit keys
// (orderable fitness << 32 | member index) below its own.  Keys are unique, so the ranks are
// exactly those of a stable sort, and the count needs no sort at all: a workgroup stages the
// orderable words of the whole population in LDS (at most 16 KB) and ranks 16 members, sixteen
// lanes per member, each lane comparing against every sixteenth key (consecutive LDS words for
// the sixteen lanes, the same words for the four members of a wavefront: no bank conflicts).
// pop / 16 workgroups run side by side, so the stage costs a few microseconds at any pop.
constexpr int kRankThreads = 256;
constexpr int kRankMembers = 16;

// The members of one block of sixteen: ord holds the orderable words of the whole population (LDS).
__device__ __forceinline__ void rank_members(const uint32_t* ord, const float* fitness, int pop, int shaping, int block,
                                             uint32_t* rank_out, float* shaped_out) {
  const int tid = threadIdx.x;
  const int part = tid & 15;
  const int m = block * kRankMembers + (tid >> 4);
  const int mc = min(m, pop - 1);
  const uint64_t key_m = (static_cast<uint64_t>(ord[mc]) << 32) | static_cast<uint32_t>(mc);
  uint32_t count = 0;
#pragma unroll 8
  for (int j = part; j < pop; j += 16) {
    const uint64_t key_j = (static_cast<uint64_t>(ord[j]) << 32) | static_cast<uint32_t>(j);
    count += key_j < key_m ? 1u : 0u;
  }
  // sum over the sixteen lanes of the member (integer adds: any order gives the same count)
  count += __shfl_xor(count, 1, 64);
  count += __shfl_xor(count, 2, 64);
  count += __shfl_xor(count, 4, 64);
  count += __shfl_xor(count, 8, 64);
  if (part == 0 && m < pop) {
    if (rank_out) rank_out[m] = count;
    if (shaped_out) {
      // one correctly rounded divide of two exactly representable integers
      const float c = static_cast<float>(2 * static_cast<int>(count) - (pop - 1)) / static_cast<float>(2 * (pop - 1));
      shaped_out[m] = shaping ? c : fitness[m];
    }
  }
}

__global__ __launch_bounds__(kRankThreads) void rank_kernel(const float* __restrict__ fitness, int pop, int shaping,
                                                            uint32_t* __restrict__ rank_out,
                                                            float* __restrict__ shaped_out) {
  __shared__ uint32_t ord[EVO_POP_MAX];
  const int tid = threadIdx.x;
  for (int i = tid; i < pop; i += kRankThreads) ord[i] = orderable(fitness[i]);
  __syncthreads();
  rank_members(ord, fitness, pop, shaping, blockIdx.x, rank_out, shaped_out);
}

// ---- tell --------------------------------------------------------------------------------
struct TellArgs {
  float* mu;
  float* sigma;
  float* m;
  float* v;
  float* ms;  // sigma moments (rule 1) or null
  float* vs;
  float* gmu_out;  // gradient-only mode
  float* gsg_out;
  const float* shaped;  // utilities c[pop] (centered ranks or raw fitness)
  const float* theta;   // stored population [2N][P] (STORED form) or null
  int P, nquads, N, KS;
  uint32_t gen, key0, key1;
  const uint32_t* gen_dev;  // when set: t is read here and the bias corrections are formed in the kernel
  float inv_n, lr_mu, lr_sigma, max_change, beta1, beta2, eps, bc1, bc2, momentum;
};

__device__ __forceinline__ float adam_step(float x, float g, float& m, float& v, float lr, const TellArgs& a) {
  m = a.beta1 * m + (1.0f - a.beta1) * g;
  v = a.beta2 * v + (1.0f - a.beta2) * g * g;
  const float m_hat = m * a.bc1;
  const float v_hat = v * a.bc2;
  return x + lr * m_hat / (sqrtf(v_hat) + a.eps);
}

// Thread (q, ks): parameter quad q, pairs ks, ks+KS, ks+2KS, ...  The KS partial sums of a
// quad are added in increasing ks by one thread, so the result does not depend on timing.
// OPT: what happens to mu.  SRULE: sigma rule 0 (clipped ascent) or 1 (Adam); unused with OPT_GRAD.
// STORED: the perturbation eps = theta[2k] - mu is read back from the population that ask wrote
// (sums of w eps and u (eps^2 - sigma^2)) instead of being regenerated (sums of w z and u (z^2 - 1)).
enum { OPT_ADAM = 0, OPT_CLIPUP_GRAD = 1, OPT_MOMENTUM = 2, OPT_GRAD = 3 };
template <int OPT, int SRULE, bool STORED>
__device__ __forceinline__ void tell_block(TellArgs a, int block, float* smem) {
  float* w_s = smem;
  float* u_s = smem + a.N;
  float* part = smem + 2 * a.N;  // [KS][QPB][8] when KS > 1
  const int tid = threadIdx.x;
  if (a.gen_dev) {  // generation index on the device: the same double-precision bias corrections the host forms
    a.gen = *a.gen_dev;
    const double t = static_cast<double>(a.gen);
    a.bc1 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(a.beta1), t)));
    a.bc2 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(a.beta2), t)));
  }
  const int QPB = 256 / a.KS;
  const int ql = tid % QPB;
  const int ks = tid / QPB;
  const int q = block * QPB + ql;
  // pair weights from the utilities: b = mean(c) in fp64 with a fixed tree (every workgroup
  // computes the same bits), w_k = (c[2k] - c[2k+1]) / 2, u_k = (c[2k] + c[2k+1]) / 2 - b
  {
    double* red = reinterpret_cast<double*>(part);  // 256 doubles: fits the partial-sum area or its minimum
    double acc = 0.0;
    for (int i = tid; i < 2 * a.N; i += 256) acc += static_cast<double>(a.shaped[i]);
    red[tid] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
      if (tid < s) red[tid] += red[tid + s];
      __syncthreads();
    }
    const double b = red[0] / static_cast<double>(2 * a.N);
    for (int k = tid; k < a.N; k += 256) {
      const double cp = a.shaped[2 * k], cm = a.shaped[2 * k + 1];
      w_s[k] = static_cast<float>(0.5 * (cp - cm));
      u_s[k] = static_cast<float>(0.5 * (cp + cm) - b);
    }
    __syncthreads();
  }
  float A[4] = {0.f, 0.f, 0.f, 0.f}, B[4] = {0.f, 0.f, 0.f, 0.f};
  if (q < a.nquads && !STORED) {
    for (int k = ks; k < a.N; k += a.KS) {
      float z[4];
      philox_normal4(static_cast<uint32_t>(q), static_cast<uint32_t>(k), a.gen, EVO_TAG_NOISE, a.key0, a.key1, z);
      const float wk = w_s[k], uk = u_s[k];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        A[i] = fmaf(wk, z[i], A[i]);
        B[i] = fmaf(uk, fmaf(z[i], z[i], -1.0f), B[i]);
      }
    }
  }
  if (q < a.nquads && STORED) {
    const int col = q * 4;
    const bool vec = (a.P & 3) == 0;  // rows are 16-byte aligned only then
    float mu4[4], nv4[4];             // centre and -sigma^2
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = min(col + i, a.P - 1);
      const float sg = a.sigma[c];
      mu4[i] = a.mu[c];
      nv4[i] = -sg * sg;
    }
#pragma unroll 8
    for (int k = ks; k < a.N; k += a.KS) {
      const float* row = a.theta + static_cast<size_t>(2 * k) * a.P;
      float th[4];
      if (vec) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + col));
        th[0] = t[0], th[1] = t[1], th[2] = t[2], th[3] = t[3];
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) th[i] = row[min(col + i, a.P - 1)];
      }
      const float wk = w_s[k], uk = u_s[k];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = th[i] - mu4[i];
        A[i] = fmaf(wk, e, A[i]);
        B[i] = fmaf(uk, fmaf(e, e, nv4[i]), B[i]);
      }
    }
  }
  if (a.KS > 1) {
    float* mine = part + (static_cast<size_t>(ks) * QPB + ql) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mine[i] = A[i];
      mine[4 + i] = B[i];
    }
    __syncthreads();
    if (ks == 0) {
      for (int s = 1; s < a.KS; ++s) {
        const float* other = part + (static_cast<size_t>(s) * QPB + ql) * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          A[i] += other[i];
          B[i] += other[4 + i];
        }
      }
    }
  }
  if (ks != 0 || q >= a.nquads) return;
  const int col = q * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = col + i;
    if (c >= a.P) break;
    const float sg = a.sigma[c];
    const float g_mu = STORED ? A[i] * a.inv_n : sg * A[i] * a.inv_n;
    const float g_sg = STORED ? (sg > 0.f ? B[i] / sg * a.inv_n : 0.f) : sg * B[i] * a.inv_n;
    if (OPT == OPT_GRAD) {
      a.gmu_out[c] = g_mu;
      a.gsg_out[c] = g_sg;
      continue;
    }
    if (OPT == OPT_ADAM) {
      float m = a.m[c], v = a.v[c];
      a.mu[c] = adam_step(a.mu[c], g_mu, m, v, a.lr_mu, a);
      a.m[c] = m;
      a.v[c] = v;
    } else if (OPT == OPT_MOMENTUM) {
      const float vel = a.momentum * a.m[c] + a.lr_mu * g_mu;
      a.m[c] = vel;
      a.mu[c] += vel;
    } else {
      a.v[c] = g_mu;  // ClipUp needs |g_mu| over all of P first: the gradient waits in v
    }
    if (SRULE == 0) {
      const float lim = a.max_change * sg;
      a.sigma[c] = sg + fminf(fmaxf(a.lr_sigma * g_sg, -lim), lim);
    } else {
      float ms = a.ms[c], vs = a.vs[c];
      a.sigma[c] = fmaxf(adam_step(sg, g_sg, ms, vs, a.lr_sigma, a), 1e-8f);
      a.ms[c] = ms;
      a.vs[c] = vs;
    }
  }
}

template <int OPT, int SRULE, bool STORED>
__global__ __launch_bounds__(256) void tell_kernel(TellArgs a) {
  extern __shared__ float smem[];
  tell_block<OPT, SRULE, STORED>(a, blockIdx.x, smem);
}

// ---- one whole generation in one launch (small problems) ----------------------------------------------------
// ask -> forward + loss -> fitness -> ranks -> tell for problems whose five launches are bound by launch latency
// (Section 2's loop of ask, evaluate, tell at cfg1's size).  Workgroup (tile, member): draws the member's parameters
// into LDS exactly as ask_kernel would store them, runs mlp_f32_body on its tile of samples and hands the tile's
// loss sum over.  The first n_tell workgroups then wait for every tile's sum (every other workgroup exits, so those
// that wait cannot keep anyone from arriving; the wait is bounded), form every member's fitness and utility in LDS
// with the arithmetic of finalize_kernel and rank_kernel and run tell_block for their block of parameters: the
// same bits as the five launches give.  mu and sigma are first written after every workgroup has read them.
//
// The hand-over has no counter and no fence: on this chip a release at device scope writes a die's cache back
// (measured: 5 us from the end of the forward to the counted arrival, 13 us until 512 arrivals had been seen).
// The sums themselves are the flags.  There are two arrays of them, used by even and odd generations; a word
// holds kNotYet until its workgroup stores its sum with one device-scope store, the waiting workgroups poll the
// words with device-scope loads, and every workgroup re-arms its word of the OTHER array, which the previous
// launch has finished with and the next one will use.  (A sum that happened to have kNotYet's bits, one pattern
// among the NaNs, is stored as the default NaN.)
struct GenSmallArgs {
  MlpArgs mlp;       // params and partial unused: the parameters are drawn here, the sums go through `sums`
  TellArgs tell;     // shaped unused: the utilities are formed here
  float* fitness;    // [pop] out
  float scale;       // fitness = scale * sum of the member's loss sums
  uint32_t* sums;    // [2][kSmallMaxTiles] loss sums of (member, tile) as bit patterns, by parity of the generation
  uint32_t* done;    // waiting workgroups that have finished (the last one clears it and advances gen_rw)
  uint32_t* gen_rw;  // the device copy of t, or null
  int pop, shaping, n_tell, total;
};
constexpr int kSmallMaxTiles = 4096;       // (member, tile) pairs of one launch
constexpr uint32_t kNotYet = 0x7fc5a5a5u;  // a quiet NaN that no arithmetic produces
constexpr int kSmallSpinLimit = 1 << 21;   // polls of about a microsecond: a sum that has not come by then never will
typedef __attribute__((address_space(3))) const float* lds_cfloat_ptr;

template <int LOSS, int OPT, int SRULE>
__global__ __launch_bounds__(256) void generation_small_kernel(GenSmallArgs g) {
  extern __shared__ __attribute__((aligned(16))) float gs_smem[];
  __shared__ int missing;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int member = blockIdx.y, tile = blockIdx.x;
  const int wg = member * gridDim.x + tile;
  const int P = g.tell.P, nquads = g.tell.nquads;
  const uint32_t gen = g.tell.gen_dev ? *g.tell.gen_dev : g.tell.gen;
  uint32_t* mine = g.sums + (gen & 1u) * kSmallMaxTiles;
  if (tid == 0) {
    missing = 0;
    __hip_atomic_store(g.sums + ((gen & 1u) ^ 1u) * kSmallMaxTiles + wg, kNotYet, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // ---- ask: this member's row, as ask_kernel forms it ----
  {
    const float sign = (member & 1) ? -1.0f : 1.0f;
    for (int q = tid; q < nquads; q += 256) {
      const int col = q * 4;
      float mu4[4], sg4[4];
      if (col + 3 < P) {
        const float4 a = *reinterpret_cast<const float4*>(g.tell.mu + col);
        const float4 b = *reinterpret_cast<const float4*>(g.tell.sigma + col);
        mu4[0] = a.x, mu4[1] = a.y, mu4[2] = a.z, mu4[3] = a.w;
        sg4[0] = b.x, sg4[1] = b.y, sg4[2] = b.z, sg4[3] = b.w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          mu4[i] = col + i < P ? g.tell.mu[col + i] : 0.f;
          sg4[i] = col + i < P ? g.tell.sigma[col + i] : 0.f;
        }
      }
      float z[4];
      philox_normal4(static_cast<uint32_t>(q), static_cast<uint32_t>(member >> 1), gen, EVO_TAG_NOISE, g.tell.key0,
                     g.tell.key1, z);
#pragma unroll
      for (int i = 0; i < 4; ++i) gs_smem[col + i] = fmaf(sign * sg4[i], z[i], mu4[i]);
    }
  }
  __syncthreads();
  // ---- forward and loss of this tile; thread 0 holds the tile's sum and hands it over ----
  float* mlp_lds = gs_smem + 4 * nquads;
  const float tile_loss = mlp_f32_body<LOSS>(g.mlp, (lds_cfloat_ptr)gs_smem, member, tile, mlp_lds);
  if (tid == 0) {
    uint32_t bits = __float_as_uint(tile_loss);
    if (bits == kNotYet) bits = 0x7fc00000u;
    __hip_atomic_store(mine + wg, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (wg >= g.n_tell) return;
  __syncthreads();  // the tile's LDS is free
  // ---- every tile's sum, polled into LDS ----
  float* fit_s = gs_smem;
  float* shaped_s = fit_s + g.pop;
  uint32_t* ord_s = reinterpret_cast<uint32_t*>(shaped_s + g.pop);
  float* part_s = reinterpret_cast<float*>(ord_s + g.pop);
  float* tell_smem = part_s + g.total;
  for (int i = tid; i < g.total; i += 256) {
    uint32_t bits = __hip_atomic_load(mine + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int polls = 0; bits == kNotYet && polls < kSmallSpinLimit; ++polls) {
      __builtin_amdgcn_s_sleep(2);
      bits = __hip_atomic_load(mine + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (bits == kNotYet) missing = 1;
    part_s[i] = __uint_as_float(bits);
  }
  __syncthreads();
  if (missing) {  // never seen; the fitness says so rather than a silent wrong update
    if (wg == 0 && tid == 0) g.fitness[0] = __builtin_nanf("");
    return;
  }
  // ---- fitness, orderable words and utilities of every member, in LDS ----
  // finalize_kernel's sum per member: lane j takes tiles j, j + 64, ..., then the fixed butterfly over the 64 lanes.
  // With at most 16 tiles the butterfly's first two levels add the zeros of lanes 16..63 (x + 0 = x, and a sum of
  // per-sample losses is never -0), so four members share a wave, sixteen lanes each, and take the last four levels.
  const int tiles = g.mlp.tiles;
  if (tiles <= 16) {
    const int sub = lane >> 4, j = lane & 15;
    for (int m0 = 4 * wave; m0 < g.pop; m0 += 16) {
      const int m = m0 + sub;
      float acc = (m < g.pop && j < tiles) ? part_s[m * tiles + j] : 0.f;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
      if (j == 0 && m < g.pop) {
        const float f = g.scale * acc;
        fit_s[m] = f;
        if (wg == 0) g.fitness[m] = f;
      }
    }
  } else {
    for (int m = wave; m < g.pop; m += 4) {
      float acc = 0.f;
      for (int j = lane; j < tiles; j += 64) acc += part_s[m * tiles + j];
      acc = wave_sum(acc);
      if (lane == 0) {
        const float f = g.scale * acc;
        fit_s[m] = f;
        if (wg == 0) g.fitness[m] = f;
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < g.pop; i += 256) ord_s[i] = orderable(fit_s[i]);
  __syncthreads();
  for (int blk = 0; blk * kRankMembers < g.pop; ++blk) rank_members(ord_s, fit_s, g.pop, g.shaping, blk, nullptr, shaped_s);
  __syncthreads();
  // ---- tell for this workgroup's block of parameters ----
  TellArgs a = g.tell;
  a.shaped = shaped_s;
  tell_block<OPT, SRULE, false>(a, wg, tell_smem);
  if (g.gen_rw == nullptr) return;
  __syncthreads();
  if (tid == 0) {  // t on the device: the last of the waiting workgroups to finish advances it
    if (atomicAdd(g.done, 1u) == static_cast<uint32_t>(g.n_tell - 1)) {
      *g.done = 0u;
      *g.gen_rw += 1u;
    }
  }
}

// ---- ClipUp: two norms over P, each as kNormBlocks partial sums in a fixed order ------------------
// Sum of the 256 per-thread values of a workgroup, fixed tree; valid in thread 0.
__device__ __forceinline__ float block_sum256(float v, float* scratch) {
  scratch[threadIdx.x] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) scratch[threadIdx.x] += scratch[threadIdx.x + s];
    __syncthreads();
  }
  return scratch[0];
}

// Total of kNormBlocks partial sums in increasing order, fp64; every thread gets the same bits.
__device__ __forceinline__ double partials_total(const float* __restrict__ part, double* scratch) {
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kNormBlocks; ++i) t += static_cast<double>(part[i]);
    scratch[0] = t;
  }
  __syncthreads();
  return scratch[0];
}

// part[b] = sum of x[i]^2 over the elements of workgroup b (grid-stride, kNormBlocks workgroups).
__global__ __launch_bounds__(256) void sqnorm_kernel(const float* __restrict__ x, int P, float* __restrict__ part) {
  __shared__ float scratch[256];
  float acc = 0.f;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < P; i += kNormBlocks * 256) acc = fmaf(x[i], x[i], acc);
  const float t = block_sum256(acc, scratch);
  if (threadIdx.x == 0) part[blockIdx.x] = t;
}

// vel = momentum vel + step g / |g| (g waits in `g`, |g|^2 in part_g); partial sums of vel^2 to part_v.
__global__ __launch_bounds__(256) void clipup_velocity_kernel(float* __restrict__ vel, const float* __restrict__ g,
                                                              int P, float momentum, float step,
                                                              const float* __restrict__ part_g,
                                                              float* __restrict__ part_v) {
  __shared__ float scratch[256];
  __shared__ double total[1];
  const double n2 = partials_total(part_g, total);
  const float scale = n2 > 0.0 ? static_cast<float>(static_cast<double>(step) / sqrt(n2)) : 0.f;
  float acc = 0.f;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < P; i += kNormBlocks * 256) {
    const float v = fmaf(scale, g[i], momentum * vel[i]);
    vel[i] = v;
    acc = fmaf(v, v, acc);
  }
  const float t = block_sum256(acc, scratch);
  if (threadIdx.x == 0) part_v[blockIdx.x] = t;
}

// Clip the velocity to max_speed and move mu.
__global__ __launch_bounds__(256) void clipup_apply_kernel(float* __restrict__ mu, float* __restrict__ vel, int P,
                                                           float max_speed, const float* __restrict__ part_v) {
  __shared__ double total[1];
  const double speed = sqrt(partials_total(part_v, total));
  const float clip = speed > static_cast<double>(max_speed) ? static_cast<float>(static_cast<double>(max_speed) / speed) : 1.0f;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < P; i += kNormBlocks * 256) {
    const float v = vel[i] * clip;
    vel[i] = v;
    mu[i] += v;
  }
}

// rows copies of the centre: params[r][i] = mu[i] (fp32) or its bfloat16 rounding.
template <typename OutT>
__global__ __launch_bounds__(256) void center_kernel(const float* __restrict__ mu, OutT* __restrict__ params, int P,
                                                     int rows) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= P) return;
  const float v = mu[i];
  for (int r = 0; r < rows; ++r) {
    if (sizeof(OutT) == 4) reinterpret_cast<float*>(params)[static_cast<size_t>(r) * P + i] = v;
    else reinterpret_cast<uint16_t*>(params)[static_cast<size_t>(r) * P + i] = to_bf16(v);
  }
}

// t <- value (set != 0) or t <- t + 1, by one thread, in stream order after the kernels that read t.
__global__ void generation_kernel(uint32_t* __restrict__ gen, uint32_t value, int set) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *gen = set ? value : *gen + 1u;
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, size_t n, float value) {
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) p[i] = value;
}

static int fill(float* p, size_t n, float value, hipStream_t s) {
  if (n == 0) return EVO_OK;
  const unsigned blocks = static_cast<unsigned>(n / 256 + 1 < 4096 ? n / 256 + 1 : 4096);
  hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, s, p, n, value);
  return check_launch("fill_kernel");
}

__global__ __launch_bounds__(256) void philox_words_kernel(uint32_t gen, uint32_t pair, uint32_t block0,
                                                           uint32_t nblocks, uint32_t tag, uint32_t key0,
                                                           uint32_t key1, uint32_t* __restrict__ words,
                                                           float* __restrict__ normals) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= nblocks) return;
  if (words) {
    const u32x4 w = philox4x32_10(block0 + i, pair, gen, tag, key0, key1);
    reinterpret_cast<uint4*>(words)[i] = make_uint4(w.x, w.y, w.z, w.w);
  }
  if (normals) {
    float z[4];
    philox_normal4(block0 + i, pair, gen, tag, key0, key1, z);
    reinterpret_cast<float4*>(normals)[i] = make_float4(z[0], z[1], z[2], z[3]);
  }
}

static int launch_rank(const float* fitness, int pop, int shaping, uint32_t* rank, float* shaped, hipStream_t s) {
  hipLaunchKernelGGL(rank_kernel, dim3((pop + kRankMembers - 1) / kRankMembers), dim3(kRankThreads), 0, s, fitness,
                     pop, shaping, rank, shaped);
  return check_launch("rank_kernel");
}

static int check_cfg(const pgpe_config* c) {
  EVO_REQUIRE(c != nullptr, EVO_ERR_ARG, "pgpe_config is null");
  EVO_REQUIRE(c->P >= 1, EVO_ERR_ARG, "P must be >= 1 (got %d)", c->P);
  EVO_REQUIRE(c->pop_max >= 2 && c->pop_max <= EVO_POP_MAX && (c->pop_max & 1) == 0, EVO_ERR_ARG,
              "pop_max must be even and in [2, %d] (got %d)", EVO_POP_MAX, c->pop_max);
  EVO_REQUIRE(c->sigma_rule == 0 || c->sigma_rule == 1, EVO_ERR_ARG, "sigma_rule must be 0 or 1");
  EVO_REQUIRE(c->shaping == 0 || c->shaping == 1, EVO_ERR_ARG, "shaping must be 0 or 1");
  EVO_REQUIRE(c->beta1 >= 0.f && c->beta1 < 1.f && c->beta2 >= 0.f && c->beta2 < 1.f, EVO_ERR_ARG,
              "Adam betas must lie in [0,1)");
  EVO_REQUIRE(c->optimizer == EVO_OPT_ADAM || c->optimizer == EVO_OPT_CLIPUP || c->optimizer == EVO_OPT_MOMENTUM,
              EVO_ERR_ARG, "optimizer must be EVO_OPT_ADAM, EVO_OPT_CLIPUP or EVO_OPT_MOMENTUM (got %d)", c->optimizer);
  if (c->optimizer != EVO_OPT_ADAM)
    EVO_REQUIRE(c->momentum >= 0.f && c->momentum < 1.f, EVO_ERR_ARG, "momentum must lie in [0,1)");
  if (c->optimizer == EVO_OPT_CLIPUP) EVO_REQUIRE(c->max_speed > 0.f, EVO_ERR_ARG, "max_speed must be positive");
  return EVO_OK;
}

extern "C" float pgpe_clipup_default_max_speed(float lr_mu) { return 2.0f * lr_mu; }

extern "C" int pgpe_config_defaults(pgpe_config* cfg, int32_t P, int32_t pop_max) {
  EVO_REQUIRE(cfg != nullptr, EVO_ERR_ARG, "pgpe_config_defaults: cfg is null");
  cfg->P = P, cfg->pop_max = pop_max;
  cfg->sigma_init = 0.1f, cfg->lr_mu = 0.01f, cfg->lr_sigma = 0.1f, cfg->sigma_max_change = 0.2f;
  cfg->beta1 = 0.9f, cfg->beta2 = 0.999f, cfg->eps = 1e-8f;
  cfg->sigma_rule = 0, cfg->shaping = 1, cfg->optimizer = EVO_OPT_ADAM;
  cfg->momentum = 0.9f, cfg->max_speed = pgpe_clipup_default_max_speed(cfg->lr_mu);
  return EVO_OK;
}

static int check_ask_pop(const pgpe_state* st, int32_t pop, const char* who) {
  EVO_REQUIRE(pop >= 2 && (pop & 1) == 0 && pop <= st->cfg.pop_max, EVO_ERR_ARG,
              "%s: pop must be even and in [2, pop_max=%d] (got %d)", who, st->cfg.pop_max, pop);
  return EVO_OK;
}

// The device copy of t, or null while the state keeps t on the host only.
static const uint32_t* device_generation(const pgpe_state* st) {
  return st->device_t ? ws_carve(st->work, st->cfg.pop_max).gen : nullptr;
}

// What the calls that fuse ask into an evaluation (other source files) need of a state.
int pgpe_view(const pgpe_state* st, PgpeView* out) {
  EVO_REQUIRE(st != nullptr && out != nullptr, EVO_ERR_ARG, "pgpe state is null");
  out->mu = st->mu, out->sigma = st->sigma, out->P = st->cfg.P, out->t = st->t;
  out->gen_dev = device_generation(st);
  return EVO_OK;
}
int pgpe_check_ask(const pgpe_state* st, int32_t pop, const char* who) { return check_ask_pop(st, pop, who); }
void pgpe_note_ask(pgpe_state* st, uint64_t seed, int32_t pop) {
  st->pending = true;
  st->seed = seed;
  st->pop = pop;
}

// Host t -> device copy, in stream order.
static int write_device_generation(pgpe_state* st, hipStream_t s) {
  hipLaunchKernelGGL(generation_kernel, dim3(1), dim3(64), 0, s, ws_carve(st->work, st->cfg.pop_max).gen, st->t, 1);
  return check_launch("generation_kernel");
}

// Device copy -> host t; waits for the stream.
static int read_device_generation(pgpe_state* st, hipStream_t s) {
  uint32_t t = 0;
  hipError_t e = hipMemcpyAsync(&t, ws_carve(st->work, st->cfg.pop_max).gen, sizeof(t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "reading the generation index back failed: %s", hipGetErrorString(e));
  st->t = t;
  return EVO_OK;
}

// After a tell: t <- t + 1, on the host and (in stream order) on the device.
static int advance_generation(pgpe_state* st, hipStream_t s) {
  st->pending = false;
  st->t += 1;
  if (!st->device_t) return EVO_OK;
  hipLaunchKernelGGL(generation_kernel, dim3(1), dim3(64), 0, s, ws_carve(st->work, st->cfg.pop_max).gen, 0u, 0);
  return check_launch("generation_kernel");
}

// The arguments of the tell kernels for the pending ask (theta: stored population or null), the number of
// workgroups and their dynamic LDS.
static TellArgs tell_args(const pgpe_state* st, float* gmu, float* gsg, const float* theta, unsigned* blocks_out,
                          size_t* shmem_out) {
  const pgpe_config& c = st->cfg;
  const int N = st->pop / 2, P = c.P;
  Workspace ws = ws_carve(st->work, c.pop_max);
  TellArgs a;
  a.mu = st->mu, a.sigma = st->sigma, a.m = st->m, a.v = st->v;
  a.ms = st->aux, a.vs = st->aux ? st->aux + P : nullptr;
  a.gmu_out = gmu, a.gsg_out = gsg;
  a.shaped = ws.shaped;
  a.theta = theta;
  a.P = P, a.nquads = (P + 3) / 4, a.N = N;
  // split the pair loop KS ways until about 2^19 threads (eight waves per SIMD) are in flight:
  // measured, that is where the time stops falling, and beyond 64 slices the LDS reduction of
  // the partial sums costs more than it gains
  int KS = 1;
  const long threads_wanted = theta ? 262144 : 524288;
  while (KS < 64 && KS * 2 <= N && static_cast<long>(a.nquads) * KS < threads_wanted) KS *= 2;
  a.KS = KS;
  a.gen = st->t, a.key0 = static_cast<uint32_t>(st->seed), a.key1 = static_cast<uint32_t>(st->seed >> 32);
  a.gen_dev = st->device_t ? ws.gen : nullptr;
  a.inv_n = 1.0f / static_cast<float>(N);
  a.lr_mu = c.lr_mu, a.lr_sigma = c.lr_sigma, a.max_change = c.sigma_max_change;
  a.beta1 = c.beta1, a.beta2 = c.beta2, a.eps = c.eps, a.momentum = c.momentum;
  a.bc1 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(c.beta1), static_cast<double>(st->t))));
  a.bc2 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(c.beta2), static_cast<double>(st->t))));
  const int QPB = 256 / KS;
  *blocks_out = static_cast<unsigned>((a.nquads + QPB - 1) / QPB);
  *shmem_out = sizeof(float) * (2 * static_cast<size_t>(N) + 256 * 8);  // w, u, partial sums / mean tree
  return a;
}

// Shared by pgpe_tell, pgpe_tell_stored and the gradient hook (theta: stored population or null).
static int run_tell(pgpe_state* st, const float* fitness, float* gmu, float* gsg, const float* theta,
                    hipStream_t s) {
  const pgpe_config& c = st->cfg;
  const int pop = st->pop, P = c.P;
  Workspace ws = ws_carve(st->work, c.pop_max);
  int rc = launch_rank(fitness, pop, c.shaping, ws.rank, ws.shaped, s);
  if (rc) return rc;
  unsigned blocks;
  size_t shmem;
  const TellArgs a = tell_args(st, gmu, gsg, theta, &blocks, &shmem);
#define EVO_TELL(OPTV, SRV)                                                                          \
  do {                                                                                               \
    if (theta) hipLaunchKernelGGL((tell_kernel<OPTV, SRV, true>), dim3(blocks), dim3(256), shmem, s, a); \
    else hipLaunchKernelGGL((tell_kernel<OPTV, SRV, false>), dim3(blocks), dim3(256), shmem, s, a);  \
  } while (0)
  if (gmu) {
    EVO_TELL(OPT_GRAD, 0);
  } else if (c.optimizer == EVO_OPT_ADAM) {
    if (c.sigma_rule == 0) EVO_TELL(OPT_ADAM, 0);
    else EVO_TELL(OPT_ADAM, 1);
  } else if (c.optimizer == EVO_OPT_MOMENTUM) {
    if (c.sigma_rule == 0) EVO_TELL(OPT_MOMENTUM, 0);
    else EVO_TELL(OPT_MOMENTUM, 1);
  } else {
    if (c.sigma_rule == 0) EVO_TELL(OPT_CLIPUP_GRAD, 0);
    else EVO_TELL(OPT_CLIPUP_GRAD, 1);
  }
#undef EVO_TELL
  rc = check_launch("tell_kernel");
  if (rc || gmu || c.optimizer != EVO_OPT_CLIPUP) return rc;
  // ClipUp: |g|, velocity and its norm, clip and move; the gradient waits in v
  hipLaunchKernelGGL(sqnorm_kernel, dim3(kNormBlocks), dim3(256), 0, s, st->v, P, ws.norm);
  hipLaunchKernelGGL(clipup_velocity_kernel, dim3(kNormBlocks), dim3(256), 0, s, st->m, st->v, P, c.momentum, c.lr_mu,
                     ws.norm, ws.norm + kNormBlocks);
  hipLaunchKernelGGL(clipup_apply_kernel, dim3(kNormBlocks), dim3(256), 0, s, st->mu, st->m, P, c.max_speed,
                     ws.norm + kNormBlocks);
  return check_launch("clipup kernels");
}

// One generation in one launch (see generation_small_kernel).  The caller has validated the task; this checks what
// the kernel itself needs and leaves the state as pgpe_ask followed by pgpe_tell would.
int pgpe_generation_small(pgpe_state* st, uint64_t seed, int32_t pop, const MlpShape& sh, const float* obs,
                          int64_t obs_stride, int B, int loss, const void* target, float scale, float* fitness,
                          hipStream_t s) {
  EVO_REQUIRE(st != nullptr, EVO_ERR_ARG, "pgpe_generation: state is null");
  int rc = check_ask_pop(st, pop, "pgpe_generation");
  if (rc) return rc;
  const pgpe_config& c = st->cfg;
  EVO_REQUIRE(sh.P == c.P, EVO_ERR_ARG, "pgpe_generation: the policy has %d parameters, the state %d", sh.P, c.P);
  EVO_REQUIRE(c.optimizer != EVO_OPT_CLIPUP, EVO_ERR_UNSUPPORTED,
              "pgpe_generation: ClipUp needs norms over all parameters between its steps (use ask, rollout, tell)");
  EVO_REQUIRE(c.P <= 8192 && sh.max_width <= 256, EVO_ERR_UNSUPPORTED,
              "pgpe_generation: at most 8192 parameters and widths up to 256 (got P = %d, width %d)", c.P, sh.max_width);
  // every waiting workgroup ranks the whole population by itself: beyond a few hundred members that tail is
  // longer than the launches it saves
  EVO_REQUIRE(pop <= 512, EVO_ERR_UNSUPPORTED, "pgpe_generation: at most 512 members (got %d)", pop);
  const uint64_t seed_before = st->seed;
  const int32_t pop_before = st->pop;
  st->seed = seed, st->pop = pop;  // what tell_args reads
  GenSmallArgs g;
  unsigned n_tell;
  size_t tell_shmem;
  g.tell = tell_args(st, nullptr, nullptr, nullptr, &n_tell, &tell_shmem);
  g.mlp.sh = sh, g.mlp.params = nullptr, g.mlp.obs = obs, g.mlp.obs_stride = obs_stride, g.mlp.B = B;
  g.mlp.out = nullptr, g.mlp.target = target, g.mlp.partial = nullptr;
  g.mlp.tiles = (B + kMlpTile - 1) / kMlpTile, g.mlp.ldw = sh.max_width, g.mlp.pop = pop;
  const long total = static_cast<long>(pop) * g.mlp.tiles;
  const size_t lds_a = sizeof(float) * (4 * static_cast<size_t>(g.tell.nquads) + 2 * static_cast<size_t>(g.mlp.ldw) * kMlpTile);
  const size_t lds_c = sizeof(float) * (3 * static_cast<size_t>(pop) + static_cast<size_t>(total)) + tell_shmem;
  const size_t lds = lds_a > lds_c ? lds_a : lds_c;
  if (!(n_tell <= 128 && static_cast<long>(n_tell) <= total && total <= kSmallMaxTiles && lds <= 160 * 1024 - 64)) {
    st->seed = seed_before, st->pop = pop_before;
    EVO_REQUIRE(false, EVO_ERR_UNSUPPORTED,
                "pgpe_generation: %u update workgroups for %ld evaluation workgroups, %zu bytes of LDS: not a small problem",
                n_tell, total, lds);
  }
  static_assert(kSmallSumWords == 2 * kSmallMaxTiles, "two arrays of sums");
  Workspace ws = ws_carve(st->work, c.pop_max);
  g.done = ws.gen + 16;  // inside the 256 bytes kept for the generation word
  g.sums = ws.gen + 64;  // behind them
  if (!st->tickets_ready) {  // once per state: nothing has arrived, nobody has finished
    rc = fill(reinterpret_cast<float*>(g.done), 1, 0.f, s);
    float not_yet;  // the bit pattern as a float (moved, never computed with)
    const uint32_t not_yet_bits = kNotYet;
    memcpy(&not_yet, &not_yet_bits, sizeof(not_yet));
    if (!rc) rc = fill(reinterpret_cast<float*>(g.sums), kSmallSumWords, not_yet, s);
    if (rc) return rc;
    st->tickets_ready = true;
  }
  g.fitness = fitness, g.scale = scale;
  g.gen_rw = st->device_t ? ws.gen : nullptr;
  g.pop = pop, g.shaping = c.shaping, g.n_tell = static_cast<int>(n_tell), g.total = static_cast<int>(total);
  const dim3 grid(g.mlp.tiles, pop);
#define EVO_GEN(LOSSV, OPTV, SRV)                                                                               \
  do {                                                                                                          \
    auto kern = generation_small_kernel<LOSSV, OPTV, SRV>;                                                      \
    if (lds > 64 * 1024) {                                                                                      \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));    \
      if (e != hipSuccess) (void)hipGetLastError();                                                             \
      EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));        \
    }                                                                                                           \
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, g);                                                       \
  } while (0)
#define EVO_GEN_OPT(LOSSV)                                                                 \
  do {                                                                                     \
    if (c.optimizer == EVO_OPT_ADAM) {                                                     \
      if (c.sigma_rule == 0) EVO_GEN(LOSSV, OPT_ADAM, 0);                                  \
      else EVO_GEN(LOSSV, OPT_ADAM, 1);                                                    \
    } else {                                                                               \
      if (c.sigma_rule == 0) EVO_GEN(LOSSV, OPT_MOMENTUM, 0);                              \
      else EVO_GEN(LOSSV, OPT_MOMENTUM, 1);                                                \
    }                                                                                      \
  } while (0)
  if (loss == LOSS_CE) EVO_GEN_OPT(LOSS_CE);
  else EVO_GEN_OPT(LOSS_MSE);
#undef EVO_GEN_OPT
#undef EVO_GEN
  rc = check_launch("generation_small_kernel");
  if (rc) return rc;
  st->pending = false;  // asked and told
  st->t += 1;           // the device copy, if any, was advanced by the kernel
  return EVO_OK;
}

}  // namespace evo

using namespace evo;

extern "C" size_t pgpe_workspace_bytes(const pgpe_config* cfg) {
  if (check_cfg(cfg) != EVO_OK) return 0;
  return ws_bytes(cfg->pop_max);
}

extern "C" int pgpe_create(pgpe_state** out, const pgpe_config* cfg, float* mu_dev, float* sigma_dev,
                           float* m_dev, float* v_dev, float* aux_dev, void* work_dev) {
  EVO_REQUIRE(out != nullptr, EVO_ERR_ARG, "pgpe_create: out is null");
  *out = nullptr;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  EVO_REQUIRE(mu_dev && sigma_dev && m_dev && v_dev && work_dev, EVO_ERR_ARG,
              "pgpe_create: mu, sigma, m, v and work must be non-null");
  EVO_REQUIRE(cfg->sigma_rule == 0 || aux_dev != nullptr, EVO_ERR_ARG,
              "pgpe_create: sigma_rule 1 needs aux_dev[2P]");
  EVO_REQUIRE(aligned16(mu_dev) && aligned16(sigma_dev) && aligned16(m_dev) && aligned16(v_dev) &&
                  aligned16(work_dev) && aligned16(aux_dev),
              EVO_ERR_ARG, "pgpe_create: device pointers must be 16-byte aligned");
  pgpe_state* st = new (std::nothrow) pgpe_state;
  EVO_REQUIRE(st != nullptr, EVO_ERR_ARG, "pgpe_create: out of host memory");
  st->cfg = *cfg;
  st->mu = mu_dev, st->sigma = sigma_dev, st->m = m_dev, st->v = v_dev, st->aux = aux_dev, st->work = work_dev;
  st->t = 1, st->device_t = false, st->pending = false, st->seed = 0, st->pop = 0, st->tickets_ready = false;
  *out = st;
  return EVO_OK;
}

extern "C" int pgpe_destroy(pgpe_state* st) {
  delete st;
  return EVO_OK;
}

extern "C" int pgpe_reset(pgpe_state* st, void* stream) {
  EVO_REQUIRE(st != nullptr, EVO_ERR_ARG, "pgpe_reset: state is null");
  hipStream_t s = as_stream(stream);
  const size_t P = static_cast<size_t>(st->cfg.P);
  int rc = fill(st->sigma, P, st->cfg.sigma_init, s);
  if (!rc) rc = fill(st->m, P, 0.f, s);
  if (!rc) rc = fill(st->v, P, 0.f, s);
  if (!rc && st->aux) rc = fill(st->aux, 2 * P, 0.f, s);
  st->t = 1;
  st->pending = false;
  if (!rc && st->device_t) rc = write_device_generation(st, s);
  return rc;
}

extern "C" int pgpe_device_generation(pgpe_state* st, const uint32_t** gen_dev_out, void* stream) {
  EVO_REQUIRE(st != nullptr, EVO_ERR_ARG, "pgpe_device_generation: state is null");
  EVO_REQUIRE(!st->pending, EVO_ERR_STATE, "pgpe_device_generation: an ask is pending (call it between tell and ask)");
  st->device_t = true;
  if (gen_dev_out) *gen_dev_out = ws_carve(st->work, st->cfg.pop_max).gen;
  return write_device_generation(st, as_stream(stream));
}

extern "C" int pgpe_sync_generation(pgpe_state* st, void* stream) {
  EVO_REQUIRE(st != nullptr, EVO_ERR_ARG, "pgpe_sync_generation: state is null");
  if (!st->device_t) return EVO_OK;
  return read_device_generation(st, as_stream(stream));
}

extern "C" int pgpe_center(const pgpe_state* st, int32_t rows, void* params_dev, int32_t dtype, void* stream) {
  EVO_REQUIRE(st != nullptr && params_dev != nullptr, EVO_ERR_ARG, "pgpe_center: null argument");
  EVO_REQUIRE(rows >= 1 && rows <= EVO_POP_MAX, EVO_ERR_ARG, "pgpe_center: rows must be in [1, %d] (got %d)",
              EVO_POP_MAX, rows);
  EVO_REQUIRE(dtype == EVO_F32 || dtype == EVO_BF16, EVO_ERR_ARG, "pgpe_center: bad dtype %d", dtype);
  const int P = st->cfg.P;
  const dim3 grid(static_cast<unsigned>((P + 255) / 256));
  if (dtype == EVO_F32)
    hipLaunchKernelGGL(center_kernel<float>, grid, dim3(256), 0, as_stream(stream), st->mu,
                       static_cast<float*>(params_dev), P, rows);
  else
    hipLaunchKernelGGL(center_kernel<uint16_t>, grid, dim3(256), 0, as_stream(stream), st->mu,
                       static_cast<uint16_t*>(params_dev), P, rows);
  return check_launch("center_kernel");
}

// ---- checkpoint: header + the state arrays, in host memory ---------------------------------------
namespace {
struct StateHeader {
  char magic[8];  // "EVOPGPE1"
  uint32_t header_bytes;
  uint32_t t;
  pgpe_config cfg;
};
const char kStateMagic[8] = {'E', 'V', 'O', 'P', 'G', 'P', 'E', '1'};

size_t state_bytes(const pgpe_config& c) {
  const size_t arrays = c.sigma_rule == 1 ? 6 : 4;  // mu, sigma, m, v (+ the two sigma moments)
  return sizeof(StateHeader) + arrays * static_cast<size_t>(c.P) * sizeof(float);
}

int copy_checked(void* dst, const void* src, size_t n, hipMemcpyKind kind, hipStream_t s, const char* who) {
  hipError_t e = hipMemcpyAsync(dst, src, n, kind, s);
  if (e != hipSuccess) {
    set_error("%s: copy failed: %s", who, hipGetErrorString(e));
    return EVO_ERR_HIP;
  }
  return EVO_OK;
}
}  // namespace

extern "C" size_t pgpe_state_bytes(const pgpe_state* st) { return st ? state_bytes(st->cfg) : 0; }

extern "C" int pgpe_state_export(const pgpe_state* st, void* host_buf, size_t bytes, void* stream) {
  EVO_REQUIRE(st != nullptr && host_buf != nullptr, EVO_ERR_ARG, "pgpe_state_export: null argument");
  EVO_REQUIRE(bytes >= state_bytes(st->cfg), EVO_ERR_ARG, "pgpe_state_export: buffer of %zu bytes, %zu needed", bytes,
              state_bytes(st->cfg));
  EVO_REQUIRE(!st->pending, EVO_ERR_STATE, "pgpe_state_export: an ask is pending (export between tell and ask)");
  uint32_t t_now = st->t;
  if (st->device_t) {  // replays of a captured generation advance only the device copy
    hipError_t e = hipMemcpyAsync(&t_now, device_generation(st), sizeof(t_now), hipMemcpyDeviceToHost, as_stream(stream));
    if (e == hipSuccess) e = hipStreamSynchronize(as_stream(stream));
    EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "pgpe_state_export: %s", hipGetErrorString(e));
  }
  StateHeader h;
  memcpy(h.magic, kStateMagic, 8);
  h.header_bytes = sizeof(StateHeader);
  h.t = t_now;
  h.cfg = st->cfg;
  memcpy(host_buf, &h, sizeof(h));
  hipStream_t s = as_stream(stream);
  char* out = static_cast<char*>(host_buf) + sizeof(StateHeader);
  const size_t row = static_cast<size_t>(st->cfg.P) * sizeof(float);
  const float* arrays[6] = {st->mu, st->sigma, st->m, st->v, st->aux, st->aux ? st->aux + st->cfg.P : nullptr};
  const int n = st->cfg.sigma_rule == 1 ? 6 : 4;
  for (int i = 0; i < n; ++i)
    if (int rc = copy_checked(out + i * row, arrays[i], row, hipMemcpyDeviceToHost, s, "pgpe_state_export")) return rc;
  hipError_t e = hipStreamSynchronize(s);
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "pgpe_state_export: %s", hipGetErrorString(e));
  return EVO_OK;
}

extern "C" int pgpe_state_import(pgpe_state* st, const void* host_buf, size_t bytes, void* stream) {
  EVO_REQUIRE(st != nullptr && host_buf != nullptr, EVO_ERR_ARG, "pgpe_state_import: null argument");
  EVO_REQUIRE(bytes >= sizeof(StateHeader), EVO_ERR_ARG, "pgpe_state_import: buffer shorter than the header");
  StateHeader h;
  memcpy(&h, host_buf, sizeof(h));
  EVO_REQUIRE(memcmp(h.magic, kStateMagic, 8) == 0 && h.header_bytes == sizeof(StateHeader), EVO_ERR_ARG,
              "pgpe_state_import: not a state written by pgpe_state_export of this library version");
  EVO_REQUIRE(h.cfg.P == st->cfg.P && h.cfg.sigma_rule == st->cfg.sigma_rule, EVO_ERR_ARG,
              "pgpe_state_import: state has P = %d, sigma_rule = %d; the handle has P = %d, sigma_rule = %d", h.cfg.P,
              h.cfg.sigma_rule, st->cfg.P, st->cfg.sigma_rule);
  EVO_REQUIRE(h.t >= 1 && bytes >= state_bytes(st->cfg), EVO_ERR_ARG, "pgpe_state_import: truncated state");
  hipStream_t s = as_stream(stream);
  const char* in = static_cast<const char*>(host_buf) + sizeof(StateHeader);
  const size_t row = static_cast<size_t>(st->cfg.P) * sizeof(float);
  float* arrays[6] = {st->mu, st->sigma, st->m, st->v, st->aux, st->aux ? st->aux + st->cfg.P : nullptr};
  const int n = st->cfg.sigma_rule == 1 ? 6 : 4;
  for (int i = 0; i < n; ++i)
    if (int rc = copy_checked(arrays[i], in + i * row, row, hipMemcpyHostToDevice, s, "pgpe_state_import")) return rc;
  hipError_t e = hipStreamSynchronize(s);  // the host buffer may be released on return
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "pgpe_state_import: %s", hipGetErrorString(e));
  st->t = h.t;
  st->pending = false;
  return st->device_t ? write_device_generation(st, s) : EVO_OK;
}

extern "C" int pgpe_get_generation(const pgpe_state* st, uint32_t* t_out) {
  EVO_REQUIRE(st && t_out, EVO_ERR_ARG, "pgpe_get_generation: null argument");
  *t_out = st->t;
  return EVO_OK;
}

extern "C" int pgpe_set_generation(pgpe_state* st, uint32_t t) {
  EVO_REQUIRE(st != nullptr && t >= 1, EVO_ERR_ARG, "pgpe_set_generation: state null or t < 1");
  EVO_REQUIRE(!st->device_t, EVO_ERR_STATE,
              "pgpe_set_generation: the state keeps t on the device; use pgpe_state_import or pgpe_reset");
  st->t = t;
  st->pending = false;
  return EVO_OK;
}

extern "C" int pgpe_ask(pgpe_state* st, uint64_t seed, int32_t pop, void* params_dev, int32_t dtype,
                        void* stream) {
  EVO_REQUIRE(st != nullptr && params_dev != nullptr, EVO_ERR_ARG, "pgpe_ask: null argument");
  if (int rc = check_ask_pop(st, pop, "pgpe_ask")) return rc;
  EVO_REQUIRE(dtype == EVO_F32 || dtype == EVO_BF16, EVO_ERR_ARG, "pgpe_ask: bad dtype %d", dtype);
  EVO_REQUIRE(aligned16(params_dev), EVO_ERR_ARG, "pgpe_ask: params_dev must be 16-byte aligned");
  const int P = st->cfg.P, N = pop / 2, nquads = (P + 3) / 4;
  const int xblocks = (nquads + 255) / 256;
  // One pair per workgroup row and x fastest: consecutive workgroups write consecutive 4 KB pieces
  // of the same two rows, which is the order HBM streams best (measured: 6.7 TB/s against
  // 4.5 TB/s with 16 pairs per workgroup at P = 2^20, pop = 1024).
  const int ppb = 1;
  const dim3 grid(static_cast<unsigned>(xblocks), static_cast<unsigned>(N));
  hipStream_t s = as_stream(stream);
  const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
  const uint32_t* gen_dev = device_generation(st);
  if (dtype == EVO_F32) {
    hipLaunchKernelGGL(ask_kernel<float>, grid, dim3(256), 0, s, st->mu, st->sigma,
                       static_cast<float*>(params_dev), P, nquads, N, ppb, st->t, gen_dev, k0, k1);
  } else if ((P & 7) == 0) {
    const int noct = P / 8;
    hipLaunchKernelGGL(ask_bf16x8_kernel, dim3(static_cast<unsigned>((noct + 255) / 256), static_cast<unsigned>(N)),
                       dim3(256), 0, s, st->mu, st->sigma, static_cast<uint16_t*>(params_dev), P, noct, st->t, gen_dev,
                       k0, k1);
  } else {
    hipLaunchKernelGGL(ask_kernel<uint16_t>, grid, dim3(256), 0, s, st->mu, st->sigma,
                       static_cast<uint16_t*>(params_dev), P, nquads, N, ppb, st->t, gen_dev, k0, k1);
  }
  int rc = check_launch("ask_kernel");
  if (rc) return rc;
  st->pending = true;
  st->seed = seed;
  st->pop = pop;
  return EVO_OK;
}

extern "C" size_t pgpe_ask_sphere_workspace_bytes(const pgpe_config* cfg) {
  if (check_cfg(cfg) != EVO_OK) return 0;
  return (static_cast<size_t>(cfg->pop_max) * fused_xblocks(cfg->P) * sizeof(float) + 255) & ~size_t(255);
}

extern "C" int pgpe_ask_sphere(pgpe_state* st, uint64_t seed, int32_t pop, const float* x_star_dev,
                               float* fitness_dev, void* work_dev, void* stream) {
  EVO_REQUIRE(st && x_star_dev && fitness_dev && work_dev, EVO_ERR_ARG, "pgpe_ask_sphere: null argument");
  int rc = check_ask_pop(st, pop, "pgpe_ask_sphere");
  if (rc) return rc;
  EVO_REQUIRE(aligned16(x_star_dev) && aligned16(work_dev), EVO_ERR_ARG,
              "pgpe_ask_sphere: x_star_dev and work_dev must be 16-byte aligned");
  const int P = st->cfg.P, N = pop / 2, nquads = (P + 3) / 4, xblocks = fused_xblocks(P);
  hipStream_t s = as_stream(stream);
  float* part = static_cast<float*>(work_dev);
  const dim3 grid(static_cast<unsigned>(xblocks), static_cast<unsigned>((N + kFusedPairs - 1) / kFusedPairs));
  hipLaunchKernelGGL(ask_sphere_kernel, grid, dim3(256), 0, s, st->mu, st->sigma, x_star_dev, part, P, nquads, N,
                     xblocks, st->t, device_generation(st), static_cast<uint32_t>(seed),
                     static_cast<uint32_t>(seed >> 32));
  rc = check_launch("ask_sphere_kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(sphere_finish_kernel, dim3(static_cast<unsigned>((pop + 3) / 4)), dim3(256), 0, s, part, xblocks,
                     pop, fitness_dev);
  rc = check_launch("sphere_finish_kernel");
  if (rc) return rc;
  st->pending = true;
  st->seed = seed;
  st->pop = pop;
  return EVO_OK;
}

extern "C" int pgpe_tell(pgpe_state* st, const float* fitness_dev, void* stream) {
  EVO_REQUIRE(st != nullptr && fitness_dev != nullptr, EVO_ERR_ARG, "pgpe_tell: null argument");
  EVO_REQUIRE(st->pending, EVO_ERR_STATE, "pgpe_tell: no pending ask");
  int rc = run_tell(st, fitness_dev, nullptr, nullptr, nullptr, as_stream(stream));
  if (rc) return rc;
  return advance_generation(st, as_stream(stream));
}

extern "C" int pgpe_tell_stored(pgpe_state* st, const float* fitness_dev, const float* params_dev, void* stream) {
  EVO_REQUIRE(st && fitness_dev && params_dev, EVO_ERR_ARG, "pgpe_tell_stored: null argument");
  EVO_REQUIRE(aligned16(params_dev), EVO_ERR_ARG, "pgpe_tell_stored: params_dev must be 16-byte aligned");
  EVO_REQUIRE(st->pending, EVO_ERR_STATE, "pgpe_tell_stored: no pending ask");
  int rc = run_tell(st, fitness_dev, nullptr, nullptr, params_dev, as_stream(stream));
  if (rc) return rc;
  return advance_generation(st, as_stream(stream));
}

extern "C" int evo_pgpe_gradients(pgpe_state* st, const float* fitness_dev, float* gmu_dev, float* gsigma_dev,
                                  const float* params_dev, void* stream) {
  EVO_REQUIRE(st && fitness_dev && gmu_dev && gsigma_dev, EVO_ERR_ARG, "evo_pgpe_gradients: null argument");
  EVO_REQUIRE(st->pending, EVO_ERR_STATE, "evo_pgpe_gradients: no pending ask");
  return run_tell(st, fitness_dev, gmu_dev, gsigma_dev, params_dev, as_stream(stream));
}

extern "C" int evo_centered_rank(const float* fitness_dev, int32_t pop, uint32_t* rank_dev, float* shaped_dev,
                                 void* stream) {
  EVO_REQUIRE(fitness_dev && rank_dev && shaped_dev, EVO_ERR_ARG, "evo_centered_rank: null argument");
  EVO_REQUIRE(pop >= 2 && pop <= EVO_POP_MAX, EVO_ERR_ARG, "evo_centered_rank: pop must be in [2, %d] (got %d)",
              EVO_POP_MAX, pop);
  return launch_rank(fitness_dev, pop, 1, rank_dev, shaped_dev, as_stream(stream));
}

static int philox_hook(uint64_t seed, uint32_t gen, uint32_t pair, uint32_t block0, uint32_t nblocks, uint32_t tag,
                       uint32_t* words, float* normals, void* stream) {
  EVO_REQUIRE(words || normals, EVO_ERR_ARG, "philox hook: output pointer is null");
  EVO_REQUIRE(aligned16(words) && aligned16(normals), EVO_ERR_ARG, "philox hook: output must be 16-byte aligned");
  if (nblocks == 0) return EVO_OK;
  hipLaunchKernelGGL(philox_words_kernel, dim3((nblocks + 255) / 256), dim3(256), 0, as_stream(stream), gen, pair,
                     block0, nblocks, tag, static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), words,
                     normals);
  return check_launch("philox_words_kernel");
}

extern "C" int evo_philox_u32(uint64_t seed, uint32_t gen, uint32_t pair, uint32_t block0, uint32_t nblocks,
                              uint32_t tag, uint32_t* out_dev, void* stream) {
  return philox_hook(seed, gen, pair, block0, nblocks, tag, out_dev, nullptr, stream);
}

extern "C" int evo_philox_normal(uint64_t seed, uint32_t gen, uint32_t pair, uint32_t block0, uint32_t nblocks,
                                 uint32_t tag, float* out_dev, void* stream) {
  return philox_hook(seed, gen, pair, block0, nblocks, tag, nullptr, out_dev, stream);
}
