// Fused whole-episode cart-pole swing-up roll-out (Section 3, "Control Tasks": the task
// roll-out loop; Section 4, "Experimenting with More Tasks": reset(keys) / step with the
// state carried over the steps; all members start from identical observations).
//
// One wavefront owns one member: its policy weights sit in registers as matrix-core
// B operands for the whole episode, the 16 roll-outs of the member are the 16 rows of
// v_mfma_f32_16x16x4_f32, and the environment state of roll-out r lives in the lanes with
// lane % 16 == r.  Nothing but the final return touches HBM.
//
// Register layouts of v_mfma_f32_16x16x4_f32 (lane = 16 q + j):
//   A[row j][k = q]   one float        B[k = q][col j]   one float
//   D[row 4 q + i][col j], i = 0..3    four floats
// The contraction index inside a layer may be permuted freely as long as A and B agree;
// layer 2 uses k = (H1/4) q + s at step s so that a lane reads H1/4 consecutive floats.
#include "kernels.h"
#include "philox.h"

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct CartpoleConst {
  float g, M, m, l, b, fscale, dt, xlim;
};

struct CartpoleArgs {
  const float* params;
  int P, R, steps;
  CartpoleConst c;
  float init_scale;
  uint32_t key0, key1, gen;
  float* fitness;
  float* ret;
  float* final_state;
};

__device__ __forceinline__ float tanh_fast(float x) {
  // 1 - 2 / (e^{2x} + 1); saturates cleanly at +-1 for large |x|
  const float e = __expf(2.0f * x);
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}

__device__ __forceinline__ float act_apply(float x, int act) {
  if (act == EVO_ACT_TANH) return tanh_fast(x);
  if (act == EVO_ACT_RELU) return fmaxf(x, 0.f);
  return x;
}

struct CpState {
  float x, xd, th, thd;
};

// One explicit-Euler step from (s, sin th, cos th) under action a; returns the new state
// and its sine / cosine (needed for the reward and for the next observation).
__device__ __forceinline__ CpState cartpole_advance(const CpState& s, float sn, float cs, float a,
                                                    const CartpoleConst& c, float& sn_new, float& cs_new) {
  const float Fe = c.fscale * a - c.b * s.xd;
  const float D = 4.0f * (c.M + c.m) - 3.0f * c.m * cs * cs;
  const float xdd = (4.0f * Fe + 2.0f * c.m * c.l * s.thd * s.thd * sn - 3.0f * c.m * c.g * sn * cs) / D;
  const float thdd = 3.0f * (c.g * sn - xdd * cs) / (2.0f * c.l);
  CpState n;
  n.x = s.x + c.dt * s.xd;
  n.xd = s.xd + c.dt * xdd;
  n.th = s.th + c.dt * s.thd;
  n.thd = s.thd + c.dt * thdd;
  sincosf(n.th, &sn_new, &cs_new);
  return n;
}

constexpr int kHStride = 68;  // LDS row stride of the hidden-activation transpose buffer

template <int NT1, int NT2>  // hidden widths in tiles of 16; NT2 == 0: one hidden layer
__global__ __launch_bounds__(64) void cartpole_kernel(CartpoleArgs a, int act1, int act2, int act3) {
  constexpr int H1 = 16 * NT1, H2 = 16 * NT2;
  constexpr int KS2 = H1 / 4;  // matrix-core steps of layer 2
  __shared__ float hbuf[16 * kHStride];
  __shared__ float abuf[16];
  const int lane = threadIdx.x;
  const int j = lane & 15, q = lane >> 4;
  const int member = blockIdx.x;
  const float* theta = a.params + static_cast<size_t>(member) * a.P;

  // ---- weights -> registers (B operands) ------------------------------------------------
  float w1[2][NT1], bias1[NT1];
#pragma unroll
  for (int t = 0; t < NT1; ++t) {
    w1[0][t] = theta[q * H1 + 16 * t + j];
    w1[1][t] = (q == 0) ? theta[4 * H1 + 16 * t + j] : 0.f;
    bias1[t] = theta[5 * H1 + 16 * t + j];
  }
  const float* th2 = theta + 5 * H1 + H1;
  float w2[NT2 > 0 ? KS2 : 1][NT2 > 0 ? NT2 : 1], bias2[NT2 > 0 ? NT2 : 1];
  float w3[NT2 > 0 ? NT2 : NT1];
  float b3;
  if (NT2 > 0) {
#pragma unroll
    for (int s = 0; s < KS2; ++s)
#pragma unroll
      for (int t = 0; t < NT2; ++t) w2[s][t] = th2[(KS2 * q + s) * H2 + 16 * t + j];
#pragma unroll
    for (int t = 0; t < NT2; ++t) {
      bias2[t] = th2[H1 * H2 + 16 * t + j];
      w3[t] = th2[H1 * H2 + H2 + 16 * t + j];
    }
    b3 = th2[H1 * H2 + H2 + H2];
  } else {
#pragma unroll
    for (int t = 0; t < NT1; ++t) w3[t] = th2[16 * t + j];
    b3 = th2[H1];
  }

  float total = 0.f;  // sum of the returns of this lane's roll-outs over all passes
  for (int r0 = 0; r0 < a.R; r0 += 16) {
    const int r = r0 + j;
    const bool valid = r < a.R;
    // ---- reset: identical for every member --------------------------------------------
    float z[4];
    philox_normal4(0u, static_cast<uint32_t>(r), a.gen, EVO_TAG_RESET, a.key0, a.key1, z);
    CpState s;
    s.x = a.init_scale * z[0];
    s.xd = a.init_scale * z[1];
    s.th = a.init_scale * z[2] + 3.14159265358979323846f;
    s.thd = a.init_scale * z[3];
    float sn, cs;
    sincosf(s.th, &sn, &cs);
    float ret = 0.f;
    bool alive = true;

    for (int step = 0; step < a.steps; ++step) {
      // ---- layer 1: observation (x, x_d, cos, sin, th_d) is the A operand directly -------
      const float a0 = q == 0 ? s.x : (q == 1 ? s.xd : (q == 2 ? cs : sn));
      const float a1 = q == 0 ? s.thd : 0.f;
      float p[4] = {0.f, 0.f, 0.f, 0.f};  // partial products of the output layer
#pragma unroll
      for (int t = 0; t < NT1; ++t) {
        floatx4 acc = {bias1[t], bias1[t], bias1[t], bias1[t]};
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, w1[0][t], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, w1[1][t], acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float h = act_apply(acc[i], act1);
          if (NT2 > 0) hbuf[(4 * q + i) * kHStride + 16 * t + j] = h;
          else p[i] = fmaf(h, w3[t], p[i]);
        }
      }
      if (NT2 > 0) {
        __syncthreads();
        // ---- layer 2: lane (row j, k group q) reads KS2 consecutive activations -------------
        float a2[KS2];
        const float4* src = reinterpret_cast<const float4*>(hbuf + j * kHStride + KS2 * q);
#pragma unroll
        for (int c4 = 0; c4 < KS2 / 4; ++c4) {
          const float4 v = src[c4];
          a2[4 * c4 + 0] = v.x, a2[4 * c4 + 1] = v.y, a2[4 * c4 + 2] = v.z, a2[4 * c4 + 3] = v.w;
        }
#pragma unroll
        for (int t = 0; t < NT2; ++t) {
          floatx4 acc = {bias2[t], bias2[t], bias2[t], bias2[t]};
#pragma unroll
          for (int s2 = 0; s2 < KS2; ++s2) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[s2], w2[s2][t], acc, 0, 0, 0);
#pragma unroll
          for (int i = 0; i < 4; ++i) p[i] = fmaf(act_apply(acc[i], act2), w3[t], p[i]);
        }
      }
      // ---- output layer: sum over the 16 columns of a row group, then hand row r its action
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) p[i] += __shfl_xor(p[i], off, 64);
      }
      if (j == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) abuf[4 * q + i] = p[i];
      }
      __syncthreads();
      const float action = act_apply(abuf[j] + b3, act3);
      __syncthreads();
      // ---- environment step --------------------------------------------------------------
      float sn_n, cs_n;
      const CpState n = cartpole_advance(s, sn, cs, action, a.c, sn_n, cs_n);
      const float reward = cs_n * expf(-n.x * n.x);
      if (alive) {
        ret += reward;
        s = n;
        sn = sn_n;
        cs = cs_n;
        alive = fabsf(n.x) <= a.c.xlim;
      }
    }
    if (valid && q == 0) {
      if (a.ret) a.ret[static_cast<size_t>(member) * a.R + r] = ret;
      if (a.final_state) {
        float* f = a.final_state + (static_cast<size_t>(member) * a.R + r) * 4;
        f[0] = s.x, f[1] = s.xd, f[2] = s.th, f[3] = s.thd;
      }
    }
    total += valid ? ret : 0.f;
  }
  // ---- fitness = mean return; rows j = 0..15 of lane group q == 0, fixed butterfly --------
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) total += __shfl_xor(total, off, 64);
  if (lane == 0 && a.fitness) a.fitness[member] = total / static_cast<float>(a.R);
}

__global__ __launch_bounds__(256) void cartpole_step_kernel(CartpoleConst c, const float* __restrict__ state,
                                                            const float* __restrict__ action,
                                                            float* __restrict__ next, float* __restrict__ reward,
                                                            int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float4 v = reinterpret_cast<const float4*>(state)[i];
  CpState s{v.x, v.y, v.z, v.w};
  float sn, cs, sn_n, cs_n;
  sincosf(s.th, &sn, &cs);
  const CpState nx = cartpole_advance(s, sn, cs, action[i], c, sn_n, cs_n);
  reinterpret_cast<float4*>(next)[i] = make_float4(nx.x, nx.xd, nx.th, nx.thd);
  reward[i] = cs_n * expf(-nx.x * nx.x);
}

static CartpoleConst make_const(const float* cp) {
  return CartpoleConst{cp[0], cp[1], cp[2], cp[3], cp[4], cp[5], cp[6], cp[7]};
}

int cartpole_supported(const MlpShape& sh, int n_rollouts) {
  EVO_REQUIRE(n_rollouts >= 1 && n_rollouts <= 64, EVO_ERR_ARG, "cartpole: n_rollouts must be in [1,64] (got %d)",
              n_rollouts);
  EVO_REQUIRE(sh.dims[0] == 5 && sh.dims[sh.n_layers] == 1, EVO_ERR_ARG,
              "cartpole: the policy must map 5 observations to 1 action");
  const bool two = sh.n_layers == 3 && sh.dims[1] == sh.dims[2] &&
                   (sh.dims[1] == 16 || sh.dims[1] == 32 || sh.dims[1] == 64);
  const bool one = sh.n_layers == 2 && (sh.dims[1] == 16 || sh.dims[1] == 32 || sh.dims[1] == 64);
  EVO_REQUIRE(one || two, EVO_ERR_UNSUPPORTED,
              "cartpole: supported policies are 5-H-1 and 5-H-H-1 with H in {16, 32, 64}");
  return EVO_OK;
}

int launch_cartpole(const MlpShape& sh, const float* params, int pop, int n_rollouts, int steps, const float* cp,
                    float init_scale, uint64_t seed, uint32_t gen, float* fitness, float* ret, float* final_state,
                    hipStream_t s) {
  CartpoleArgs a;
  a.params = params, a.P = sh.P, a.R = n_rollouts, a.steps = steps;
  a.c = make_const(cp);
  EVO_REQUIRE(a.c.dt > 0.f && a.c.l > 0.f && a.c.M > 0.f && a.c.m >= 0.f, EVO_ERR_ARG,
              "cartpole: dt, length and cart mass must be positive");
  a.init_scale = init_scale;
  a.key0 = static_cast<uint32_t>(seed), a.key1 = static_cast<uint32_t>(seed >> 32), a.gen = gen;
  a.fitness = fitness, a.ret = ret, a.final_state = final_state;
  const int H = sh.dims[1];
  const int a1 = sh.act[0], a2 = sh.n_layers == 3 ? sh.act[1] : 0, a3 = sh.act[sh.n_layers - 1];
  const dim3 grid(pop), block(64);
#define EVO_CP_CASE(T1, T2)                                                                  \
  hipLaunchKernelGGL((cartpole_kernel<T1, T2>), grid, block, 0, s, a, a1, a2, a3);          \
  return check_launch("cartpole_kernel")
  if (sh.n_layers == 3) {
    if (H == 64) { EVO_CP_CASE(4, 4); }
    if (H == 32) { EVO_CP_CASE(2, 2); }
    EVO_CP_CASE(1, 1);
  }
  if (H == 64) { EVO_CP_CASE(4, 0); }
  if (H == 32) { EVO_CP_CASE(2, 0); }
  EVO_CP_CASE(1, 0);
#undef EVO_CP_CASE
}

int launch_cartpole_step(const float* cp, const float* state, const float* action, float* next, float* reward,
                         int n, hipStream_t s) {
  hipLaunchKernelGGL(cartpole_step_kernel, dim3((n + 255) / 256), dim3(256), 0, s, make_const(cp), state, action,
                     next, reward, n);
  return check_launch("cartpole_step_kernel");
}

}  // namespace evo
