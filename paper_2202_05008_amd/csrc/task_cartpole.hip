// Fused whole-episode cart-pole swing-up roll-out (Section 3, "Control Tasks": the task
// roll-out loop; Section 4, "Experimenting with More Tasks": reset(keys) / step with the
// state carried over the steps; all members start from identical observations).
//
// One workgroup owns one member; wave w owns hidden neurons 16 w .. 16 w + 15 of both hidden
// layers, whose weights sit in its registers as matrix-core operands for the whole episode.
// The 16 roll-outs of the member are the 16 rows (or columns) of a matrix tile.  Every wave
// carries the environment state of roll-out r in its lanes with lane % 16 == r and advances it
// itself (a few dozen instructions), so observations never travel between waves; only the
// hidden activations (through LDS between the layers) and the four partial sums of the output
// layer do.  Two workgroup barriers per step; nothing but the final return touches HBM.
// Several members share a SIMD (one wave each), which hides the latency of the serial
// per-step chain.
//
// Register layouts (lane = 16 q + j):
//   v_mfma_f32_16x16x4_f32    A[row j][k = q], B[k = q][col j]: one float each
//   v_mfma_f32_16x16x32_f16   A[row j][k = 8 q + e], B[k = 8 q + e][col j], e = 0..7: eight fp16 each
//   both                      D[row 4 q + i][col j], i = 0..3: four floats
//
// With two hidden layers, layer 1 is computed transposed (rows = neurons, columns = roll-outs): four of
// its inputs on the fp32 instruction, the fifth (th_d, the lane's own state) by four multiply-adds that
// also bring the bias, so that a lane ends up with four consecutive neurons of one roll-out: after the
// activation they are split into two half-precision terms (split16.h) and stored with one 8-byte LDS
// write per term.  Layer 2 (K = H) then runs on the fp16 instruction (16 cycles for 8192 multiply-adds
// against 32 cycles for 1024 of the fp32 one), three instructions per product, within a few 1e-7 of
// fp32 arithmetic, transposed as well: the lane again holds four neurons of its own roll-out, so the
// output layer is four multiply-adds, three additions and two lane swaps between the k groups.  The
// step loop is bound by the number of vector instructions a wave issues, which is what the forms
// below are chosen by (constants folded into the operands, one reciprocal serving both split terms).  Both operands carry a
// power-of-two scale that keeps them inside fp16's range whatever their magnitude: the weights of a
// wave's 16 neurons get theirs from their largest magnitude when they are loaded; activations behind
// a tanh are stored times 2^14; activations behind a ReLU or no activation get a scale per roll-out
// and step from a bound on them (sum_k max_n |W1[k][n]| |obs_k| + max_n |b1[n]|).  The factor of the
// layer-2 pre-activation and the layer-2 bias ride in the multiply-add that feeds the next
// activation.
#include "kernels.h"
#include "philox.h"
#include "split16.h"

// Every multiply-add below is written out (fmaf where one rounding is meant): with the compiler free to fuse,
// the roll-out kernel and its build with the per-step records differed in a few last bits, which the
// chaotic dynamics turn into different returns.  Written out, both builds compute the same numbers.
#pragma clang fp contract(off)

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct CartpoleConst {
  float g, M, m, l, b, fscale, dt, xlim;
  float k3_2l;   // 3 / (2 l), rounded once on the host
  float k4, k3, k2ml, k3mg;  // 4 (M + m), 3 m, 2 m l, 3 m g: binary32 products formed on the host
  float fscale4, b4;         // 4 fscale, 4 b (exact): the force enters the equations times four
};

struct CartpoleArgs {
  const float* params;
  int P, R, steps;
  CartpoleConst c;
  float init_scale;
  uint32_t key0, key1, gen;
  const uint32_t* gen_dev;  // when set, the counter word t of the reset stream is read here
  float* fitness;
  float* ret;
  float* final_state;
  float* trace;  // [pop][R][steps][12]: what every step of every roll-out actually used, or null
};

// tanh(x) = 1 - 2 / (e^{2x} + 1) on the hardware exp2 / reciprocal; saturates cleanly at +-1.
__device__ __forceinline__ float tanh_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);  // e^{2x} = 2^{2x log2 e}
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
}

__device__ __forceinline__ float act_apply(float x, int act) {
  if (act == EVO_ACT_TANH) return tanh_fast(x);
  if (act == EVO_ACT_RELU) return fmaxf(x, 0.f);
  return x;
}

// scale * tanh(x): a result wanted times scale
__device__ __forceinline__ float tanh_times(float x, float scale) {
  const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);
  return fmaf(-2.0f * scale, __builtin_amdgcn_rcpf(e + 1.0f), scale);
}
// tanh(x u + b) with k_u = 2 log2(e) u and k_b = 2 log2(e) b formed once: a pre-activation held times 1 / u
__device__ __forceinline__ float tanh_affine(float x, float k_u, float k_b) {
  const float e = __builtin_amdgcn_exp2f(fmaf(x, k_u, k_b));
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
}

// sin and cos of an angle in radians: two-term reduction by 2 pi (2 pi = hi - lo with hi the fp32
// nearest to 2 pi), then the hardware sine / cosine, which take revolutions.
__device__ __forceinline__ void sincos_fast(float th, float& s, float& c) {
  const float n = rintf(th * 0.15915494309189535f);
  float r = fmaf(n, -6.2831854820251465f, th);
  r = fmaf(n, 1.7484555e-07f, r);
  const float t = r * 0.15915494309189535f;
  s = __builtin_amdgcn_sinf(t);
  c = __builtin_amdgcn_cosf(t);
}

struct CpState {
  float x, xd, th, thd;
};

// One explicit-Euler step from (s, sin th, cos th) under action a; returns the new state
// and its sine / cosine (needed for the reward and for the next observation).
__device__ __forceinline__ CpState cartpole_advance(const CpState& s, float sn, float cs, float a,
                                                    const CartpoleConst& c, float& sn_new, float& cs_new) {
  const float D = fmaf(-cs, c.k3 * cs, c.k4);
  // the hardware reciprocal is within one ulp; D >= 4 M + m > 0
  float num = fmaf(c.fscale4, a, -(c.b4 * s.xd));  // 4 (fscale a - b x_d)
  num = fmaf(sn, s.thd * (c.k2ml * s.thd), num);
  num = fmaf(-cs, c.k3mg * sn, num);
  const float xdd = __builtin_amdgcn_rcpf(D) * num;
  const float thdd = c.k3_2l * fmaf(c.g, sn, -(cs * xdd));
  CpState n;
  n.x = fmaf(c.dt, s.xd, s.x);
  n.xd = fmaf(c.dt, xdd, s.xd);
  n.th = fmaf(c.dt, s.thd, s.th);
  n.thd = fmaf(c.dt, thdd, s.thd);
  sincos_fast(n.th, sn_new, cs_new);
  return n;
}

__device__ __forceinline__ float step_reward(float x_new, float cs_new) {
  return cs_new * __builtin_amdgcn_exp2f((-1.4426950408889634f * x_new) * x_new);  // cos(th') exp(-x'^2)
}

// Sum over the 16 lanes of a row with DPP moves (xor 1, xor 2, half-row mirror, row mirror):
// every lane of the row ends with the total; the order is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);  // row_half_mirror
  v = dpp_add<0x140>(v);  // row_mirror
  return v;
}
// Four such sums at once: lane j of a row ends with the row's total of p[j % 4].  The first two exchanges
// halve the number of live values (a lane keeps one of a pair and hands the other to its partner), so the
// whole reduction is 11 instructions instead of 16; the order of the additions is fixed.
__device__ __forceinline__ float row16_sum4(const float (&p)[4], int j) {
  const bool odd = (j & 1) != 0, upper = (j & 2) != 0;
  const float t01 = (odd ? p[1] : p[0]) +
                    __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(odd ? p[0] : p[1]), 0xB1, 0xf, 0xf, false));
  const float t23 = (odd ? p[3] : p[2]) +
                    __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(odd ? p[2] : p[3]), 0xB1, 0xf, 0xf, false));
  float u = (upper ? t23 : t01) +
            __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(upper ? t01 : t23), 0x4E, 0xf, 0xf, false));
  u = dpp_add<0x124>(u);  // row_ror:4
  u = dpp_add<0x128>(u);  // row_ror:8
  return u;
}

// NT: hidden width 16 NT (NT waves); TWO: two hidden layers of that width; TANH: every activation
// is tanh (the usual policy), which removes the per-value activation switch from the step loop.
// TRACE: the same kernel with one record per step stored to a.trace (a build of its own, because even
// a never-taken branch around the stores cost the plain roll-out 10 % of its time).
template <int NT, bool TWO, bool TANH, bool TRACE>
__global__ __launch_bounds__(64 * NT) void cartpole_kernel(CartpoleArgs a, int act1_rt, int act2_rt, int act3_rt) {
  const int act1 = TANH ? EVO_ACT_TANH : act1_rt, act2 = TANH ? EVO_ACT_TANH : act2_rt;
  const int act3 = TANH ? EVO_ACT_TANH : act3_rt;
  constexpr float kSTanh = 16384.0f;  // 2^14: scale of stored activations that a tanh bounds
  constexpr int H = 16 * NT;
  constexpr int KP = H < 32 ? 32 : H;      // contraction length of layer 2, padded to the instruction's 32
  constexpr int KS2 = KP / 32;             // matrix-core steps of layer 2 per split term pair
  constexpr int kRowB = (KP + 8) * 2;      // bytes of one roll-out's row of one term (16 bytes of padding)
  constexpr int kTermB = 16 * kRowB;       // one term of the hidden activations: [roll-out][neuron] fp16
  __shared__ __attribute__((aligned(16))) unsigned char hb[TWO ? 2 * kTermB : 16];
  __shared__ float part[NT][16];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 15, q = lane >> 4;
  const int member = blockIdx.x;
  if (a.gen_dev) a.gen = *a.gen_dev;
  const float* theta = a.params + static_cast<size_t>(member) * a.P;
  const int col = 16 * wave + j;  // this lane's hidden neuron

  // ---- weights -> registers (B operands of this wave's column tile) ----------------------------
  // With two tanh layers the first layer's weights and biases carry the factor 2 log2(e) of the tanh's
  // exp2 argument, so the pre-activations leave the product ready for the exponential.
  constexpr float kLog2e2 = 2.885390081777927f;
  const float kk = (TWO && TANH) ? kLog2e2 : 1.0f;
  const float w1a = kk * theta[q * H + col];                 // k = q      (x, x_d, cos, sin)
  const float w1b = (q == 0) ? theta[4 * H + col] : 0.f;     // k = 4 + q  (th_d, then padding): one hidden layer only
  const float bias1 = theta[5 * H + col];
  const float* th2 = theta + 5 * H + H;
  f16x8 w2b[2][TWO ? KS2 : 1];  // [term][step]: element e is s_w W2[32 step + 8 q + e][col]
  float bias1t[4], w_thd[4];     // transposed layer 1: this lane's rows are neurons 16 wave + 4 q + i
  float w3 = 0.f, b3;            // one hidden layer: output weight of this lane's column
  float bias2t[4], w3t[4];       // two: layer-2 bias and output weight of this lane's rows (neurons 16 wave + 4 q + i)
  float u_w = 1.0f;              // 1 / s_w, s_w the scale of this wave's layer-2 weights
  float bound_w[5] = {0.f, 0.f, 0.f, 0.f, 0.f}, bound_b = 0.f;  // !TANH: max_n |W1[k][n]|, max_n |b1[n]|
  if (TWO) {
    float x[KS2][8];
    float w_max = 0.f;
#pragma unroll
    for (int s = 0; s < KS2; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = 32 * s + 8 * q + e;
        x[s][e] = k < H ? th2[k * H + col] : 0.f;
        w_max = fmaxf(w_max, fabsf(x[s][e]));
      }
    const float s_w = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(wave_max(w_max)))));
    u_w = pow2_reciprocal(s_w);
#pragma unroll
    for (int s = 0; s < KS2; ++s) {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[s][e] *= s_w;
      split2_x8_true<true>(x[s], w2b[0][s], w2b[1][s]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bias1t[i] = kk * theta[5 * H + 16 * wave + 4 * q + i];
      w_thd[i] = kk * theta[4 * H + 16 * wave + 4 * q + i];  // the fifth input (th_d) is added by the vector ALU
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bias2t[i] = th2[H * H + 16 * wave + 4 * q + i];
      w3t[i] = th2[H * H + H + 16 * wave + 4 * q + i];
    }
    b3 = th2[H * H + H + H];
    // columns H .. KP - 1 of the activation rows are never written and must read as zero
    for (int i = threadIdx.x; i < 2 * kTermB / 4; i += 64 * NT) reinterpret_cast<uint32_t*>(hb)[i] = 0u;
    if (!TANH) {
      // bounds on the layer-1 pre-activations of the whole member: the largest weight per input, the largest bias
      __shared__ float wg_max[NT][6];
      float m[6];
#pragma unroll
      for (int k = 0; k < 5; ++k) m[k] = wave_max(fabsf(theta[k * H + col]));
      m[5] = wave_max(fabsf(bias1));
      if (lane == 0) {
#pragma unroll
        for (int k = 0; k < 6; ++k) wg_max[wave][k] = m[k];
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 6; ++k) {
        float v = wg_max[0][k];
#pragma unroll
        for (int w = 1; w < NT; ++w) v = fmaxf(v, wg_max[w][k]);
        if (k < 5) bound_w[k] = v; else bound_b = v;
      }
    }
    __syncthreads();
  } else {
    w3 = th2[col];
    b3 = th2[H];
  }
  // the factor 1 / (2^14 s_w) and the bias of the layer-2 pre-activation inside the tanh's exp2 argument
  const float k_u2 = kLog2e2 * (u_w * (1.0f / kSTanh));
  float k_b2t[4], m2w3t[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    k_b2t[i] = TWO ? kLog2e2 * bias2t[i] : 0.f;
    m2w3t[i] = TWO ? -2.0f * w3t[i] : 0.f;  // w3 tanh(x) = w3 - 2 w3 / (e^{2x} + 1): one multiply-add
    asm volatile("" : "+v"(m2w3t[i]));      // kept in its register (the compiler would form it again every step)
  }
  const float k_b3 = kLog2e2 * b3;    // the output tanh's argument is 2 log2(e) (sum) + this

  float total = 0.f;  // sum of the returns of this lane's roll-outs over all passes
  for (int r0 = 0; r0 < a.R; r0 += 16) {
    const int r = r0 + j;
    const bool valid = r < a.R;
    // ---- reset: identical for every member ----------------------------------------------------
    float z[4];
    philox_normal4(0u, static_cast<uint32_t>(r), a.gen, EVO_TAG_RESET, a.key0, a.key1, z);
    CpState s;
    s.x = a.init_scale * z[0];
    s.xd = a.init_scale * z[1];
    s.th = fmaf(a.init_scale, z[2], 3.14159265358979323846f);
    s.thd = a.init_scale * z[3];
    float sn, cs;
    sincos_fast(s.th, sn, cs);
    float ret = 0.f;
    bool alive = true;

    for (int step = 0; step < a.steps; ++step) {
      // ---- layer 1: observation (x, x_d, cos, sin, th_d) is the A operand directly -------------
      const float a0 = q == 0 ? s.x : (q == 1 ? s.xd : (q == 2 ? cs : sn));
      float p[4];
      if (TWO) {
        // transposed: rows = this wave's neurons, columns = roll-outs; the column of th_d is this lane's own state
        floatx4 acc;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = fmaf(w_thd[i], s.thd, bias1t[i]);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w1a, a0, acc, 0, 0, 0);
        // neurons 16 wave + 4 q .. + 3 of roll-out j: two terms, 8 bytes each
        float u_mine = 0.f;  // !TANH: 1 / (scale of the stored activations of this lane's roll-out times s_w)
        {
          float h1[4];
          uint2 lead, resid;
          if (TANH) {
#pragma unroll
            for (int i = 0; i < 4; ++i)  // 2^14 tanh
              h1[i] = fmaf(-2.0f * kSTanh, __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(acc[i]) + 1.0f), kSTanh);
            split2_pair_true(h1[0], h1[1], lead.x, resid.x);
            split2_pair_true(h1[2], h1[3], lead.y, resid.y);
          } else {
            // scale of this roll-out's activations at this step, from the bound on the pre-activations
            // (every wave carries the same state and forms the same number); a tanh bounds them by 1
            float bound = bound_b;
            bound = fmaf(bound_w[0], fabsf(s.x), bound);
            bound = fmaf(bound_w[1], fabsf(s.xd), bound);
            bound = fmaf(bound_w[2], fabsf(cs), bound);
            bound = fmaf(bound_w[3], fabsf(sn), bound);
            bound = fmaf(bound_w[4], fabsf(s.thd), bound);
            const float s_row = act1 == EVO_ACT_TANH ? kSTanh : split_pow2_scale(bound);
            u_mine = pow2_reciprocal(s_row) * u_w;
#pragma unroll
            for (int i = 0; i < 4; ++i) h1[i] = s_row * act_apply(acc[i], act1);
            split2_pair_true(h1[0], h1[1], lead.x, resid.x);
            split2_pair_true(h1[2], h1[3], lead.y, resid.y);
          }
          unsigned char* dst = hb + j * kRowB + (16 * wave + 4 * q) * 2;
          *reinterpret_cast<uint2*>(dst) = lead;
          *reinterpret_cast<uint2*>(dst + kTermB) = resid;
        }
        __syncthreads();
        // ---- layer 2, transposed as well (the weights are the row operand): lane (column j, k group q) reads 8
        //      consecutive activations of its roll-out per term and step and ends with neurons 16 wave + 4 q + i ----
        floatx4 acc2 = {0.f, 0.f, 0.f, 0.f};  // h h' + h m' + m h', the small partial products first
        const unsigned char* src = hb + j * kRowB + 16 * q;
        f16x8 at[KS2][2];
#pragma unroll
        for (int s2 = 0; s2 < KS2; ++s2)
#pragma unroll
          for (int k = 0; k < 2; ++k) at[s2][k] = *reinterpret_cast<const f16x8*>(src + k * kTermB + 64 * s2);
#pragma unroll
        for (int s2 = 0; s2 < KS2; ++s2) {
          acc2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2b[0][s2], at[s2][1], acc2, 0, 0, 0);
          acc2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2b[1][s2], at[s2][0], acc2, 0, 0, 0);
        }
#pragma unroll
        for (int s2 = 0; s2 < KS2; ++s2)
          acc2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2b[0][s2], at[s2][0], acc2, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pre = acc2[i];  // layer-2 product times the two scales
          if (TANH)
            p[i] = fmaf(m2w3t[i], __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(fmaf(pre, k_u2, k_b2t[i])) + 1.0f),
                        w3t[i]);
          else
            p[i] = act_apply(fmaf(pre, u_mine, bias2t[i]), act2) * w3t[i];
        }
        // ---- output layer: this lane's four neurons, the other twelve of the wave from the other k groups ----
        float p_wave = (p[0] + p[1]) + (p[2] + p[3]);
        {
          // register-to-register lane swaps (an exchange through LDS would put two more round trips on the step's
          // chain): lanes l and l + 32, then the 16-lane groups pairwise; every lane ends with the wave's total
          const uint32_t pb = __float_as_uint(p_wave);
          const auto h = __builtin_amdgcn_permlane32_swap(pb, pb, false, false);  // (lower, lower), (upper, upper)
          const uint32_t ph = __float_as_uint(__uint_as_float(h[0]) + __uint_as_float(h[1]));
          const auto g = __builtin_amdgcn_permlane16_swap(ph, ph, false, false);  // groups (0 0 2 2), (1 1 3 3)
          p_wave = __uint_as_float(g[0]) + __uint_as_float(g[1]);
        }
        if (q == 0) part[wave][j] = p_wave;
      } else {
        floatx4 acc = {bias1, bias1, bias1, bias1};
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, w1a, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(q == 0 ? s.thd : 0.f, w1b, acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = act_apply(acc[i], act1) * w3;
        // ---- output layer: this wave's 16 columns ----
        const float p_row = row16_sum4(p, j);  // lane j < 4: roll-out 4 q + j
        if (j < 4) part[wave][4 * q + j] = p_row;
      }
      __syncthreads();  // then the waves' partial sums in wave order
      float pre = part[0][j];
#pragma unroll
      for (int w = 1; w < NT; ++w) pre += part[w][j];
      const float lin = pre + b3;  // the policy's linear output
      const float action =
          TANH ? fmaf(-2.0f, __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(fmaf(pre, kLog2e2, k_b3)) + 1.0f), 1.0f)
               : act_apply(lin, act3);
      // ---- environment step (every wave advances its own copy of the state) -------------------
      float sn_n, cs_n;
      const CpState n = cartpole_advance(s, sn, cs, action, a.c, sn_n, cs_n);
      const float reward = step_reward(n.x, cs_n);
      if (TRACE) {
        // the state the policy saw; its linear output, the action, the step's reward, alive before; return after
        if (valid && q == 0 && wave == 0) {
          float4* tr = reinterpret_cast<float4*>(
              a.trace + ((static_cast<size_t>(member) * a.R + r) * a.steps + step) * 12);
          tr[0] = make_float4(s.x, s.xd, s.th, s.thd);
          tr[1] = make_float4(lin, action, reward, alive ? 1.f : 0.f);
          tr[2] = make_float4(alive ? ret + reward : ret, 0.f, 0.f, 0.f);
        }
      }
      if (alive) {
        ret += reward;
        s = n;
        sn = sn_n;
        cs = cs_n;
        alive = fabsf(n.x) <= a.c.xlim;
      }
      if (!TWO) __syncthreads();  // the partial sums are rewritten next step
    }
    if (valid && q == 0 && wave == 0) {
      if (a.ret) a.ret[static_cast<size_t>(member) * a.R + r] = ret;
      if (a.final_state) {
        float* f = a.final_state + (static_cast<size_t>(member) * a.R + r) * 4;
        f[0] = s.x, f[1] = s.xd, f[2] = s.th, f[3] = s.thd;
      }
    }
    total += valid ? ret : 0.f;
    __syncthreads();
  }
  // ---- fitness = mean return over the roll-outs (rows j = 0..15, fixed order) -----------------
  total = row16_sum(total);
  if (threadIdx.x == 0 && a.fitness) a.fitness[member] = total / static_cast<float>(a.R);
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
  sincos_fast(s.th, sn, cs);
  const CpState nx = cartpole_advance(s, sn, cs, action[i], c, sn_n, cs_n);
  reinterpret_cast<float4*>(next)[i] = make_float4(nx.x, nx.xd, nx.th, nx.thd);
  reward[i] = step_reward(nx.x, cs_n);
}

static CartpoleConst make_const(const float* cp) {
  const float g = cp[0], M = cp[1], m = cp[2], l = cp[3];
  return CartpoleConst{g, M, m, l, cp[4], cp[5], cp[6], cp[7], static_cast<float>(3.0 / (2.0 * static_cast<double>(l))),
                       4.0f * (M + m), 3.0f * m, (2.0f * m) * l, (3.0f * m) * g, 4.0f * cp[5], 4.0f * cp[4]};
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
                    float init_scale, uint64_t seed, uint32_t gen, const uint32_t* gen_dev, float* fitness, float* ret,
                    float* final_state, float* trace, hipStream_t s) {
  CartpoleArgs a;
  a.params = params, a.P = sh.P, a.R = n_rollouts, a.steps = steps;
  a.c = make_const(cp);
  EVO_REQUIRE(a.c.dt > 0.f && a.c.l > 0.f && a.c.M > 0.f && a.c.m >= 0.f, EVO_ERR_ARG,
              "cartpole: dt, length and cart mass must be positive");
  a.init_scale = init_scale;
  a.key0 = static_cast<uint32_t>(seed), a.key1 = static_cast<uint32_t>(seed >> 32), a.gen = gen;
  a.gen_dev = gen_dev;
  a.fitness = fitness, a.ret = ret, a.final_state = final_state, a.trace = trace;
  const int H = sh.dims[1];
  const int a1 = sh.act[0], a2 = sh.n_layers == 3 ? sh.act[1] : 0, a3 = sh.act[sh.n_layers - 1];
  const dim3 grid(pop);
  const bool all_tanh = a1 == EVO_ACT_TANH && a3 == EVO_ACT_TANH && (sh.n_layers == 2 || a2 == EVO_ACT_TANH);
#define EVO_CP_LAUNCH(NTV, TWOV, TANHV)                                                                              \
  if (trace)                                                                                                         \
    hipLaunchKernelGGL((cartpole_kernel<NTV, TWOV, TANHV, true>), grid, dim3(64 * NTV), 0, s, a, a1, a2, a3);       \
  else                                                                                                               \
    hipLaunchKernelGGL((cartpole_kernel<NTV, TWOV, TANHV, false>), grid, dim3(64 * NTV), 0, s, a, a1, a2, a3)
#define EVO_CP_CASE(NTV, TWOV)                  \
  if (all_tanh) {                               \
    EVO_CP_LAUNCH(NTV, TWOV, true);             \
  } else {                                      \
    EVO_CP_LAUNCH(NTV, TWOV, false);            \
  }                                             \
  return check_launch("cartpole_kernel")
  if (sh.n_layers == 3) {
    if (H == 64) { EVO_CP_CASE(4, true); }
    if (H == 32) { EVO_CP_CASE(2, true); }
    EVO_CP_CASE(1, true);
  }
  if (H == 64) { EVO_CP_CASE(4, false); }
  if (H == 32) { EVO_CP_CASE(2, false); }
  EVO_CP_CASE(1, false);
#undef EVO_CP_CASE
#undef EVO_CP_LAUNCH
}

int launch_cartpole_step(const float* cp, const float* state, const float* action, float* next, float* reward,
                         int n, hipStream_t s) {
  hipLaunchKernelGGL(cartpole_step_kernel, dim3((n + 255) / 256), dim3(256), 0, s, make_const(cp), state, action,
                     next, reward, n);
  return check_launch("cartpole_step_kernel");
}

}  // namespace evo
