// Population-batched MLP forward with bfloat16 weights on the matrix cores: every member
// has its own weight matrices and its own (or a shared) batch of observations (Section 2,
// "Global Policy"; Section 4, "Exploring Novel Policy Architectures").
//
// One workgroup per member.  A layer is out[B][N] = act(in[B][K] W[K][N] + b) with
// v_mfma_f32_32x32x16_bf16: activations live in LDS as bf16 rows (A operand: 8 consecutive
// k per lane, one 16-byte read), the weights stream from HBM exactly once (B operand),
// accumulation, bias and activation are fp32, and only the fitness (or the final outputs)
// is written back.  Arithmetic intensity is B flop per weight byte, so at small B the
// kernel is bound by the weight stream, not by the matrix cores.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (lane = 32 g + c):
//   A[row c][k = 8 g + i], B[k = 8 g + i][col c], i = 0..7 (eight bf16 per lane)
//   D[row 8 b + 4 g + i][col c] in register 4 b + i, b = 0..3, i = 0..3
#include <type_traits>

#include "bf16.h"
#include "kernels.h"
#include "philox.h"

namespace evo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBf16Threads = 256;
constexpr int kBf16Waves = kBf16Threads / 64;
constexpr int kMaxRows = 64;    // B <= 64: two 32-row tiles
constexpr int kMaxWidth = 256;  // widest layer
constexpr int kRowPad = 8;      // bf16 elements of padding per LDS row (16 bytes: keeps 16-byte alignment)

struct Bf16Args {
  MlpShape sh;
  const uint16_t* params;
  const float* obs;
  int64_t obs_stride;
  int B;
  float* out;
  const float* target;
  float* fitness;
  int loss;
  int buf_elems;  // bf16 elements per activation buffer
};

union Pack8 {
  uint16_t h[8];
  uint4 v;
  bf16x8 b;
};

__global__ __launch_bounds__(kBf16Threads) void mlp_bf16_kernel(Bf16Args a) {
  // two activation buffers [rows][width + pad] of bf16 (dynamic LDS, sized by the launcher)
  extern __shared__ __attribute__((aligned(16))) uint16_t act_dyn[];
  __shared__ float red[kBf16Waves];
  uint16_t* act_buf[2] = {act_dyn, act_dyn + a.buf_elems};
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 31, g = lane >> 5;
  const int member = blockIdx.x;
  const int B = a.B;
  const int m_tiles = (B + 31) / 32;
  const uint16_t* theta = a.params + static_cast<size_t>(member) * a.sh.P;
  const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;

  // ---- observations -> bf16 rows in LDS (rows beyond B are zero) ---------------------------
  {
    const int D = a.sh.dims[0], ld = D + kRowPad;
    for (int i = tid; i < m_tiles * 32 * D; i += kBf16Threads) {
      const int r = i / D, d = i - r * D;
      act_buf[0][r * ld + d] = r < B ? to_bf16(obs[static_cast<size_t>(r) * D + d]) : uint16_t(0);
    }
  }
  __syncthreads();

  int cur = 0;
  int off = 0;
  float loss_acc = 0.f;
  for (int l = 0; l < a.sh.n_layers; ++l) {
    const int K = a.sh.dims[l], N = a.sh.dims[l + 1], act = a.sh.act[l];
    const uint16_t* W = theta + off;       // [K][N]
    const uint16_t* bias = W + K * N;      // [N]
    const int ld_in = K + kRowPad, ld_out = N + kRowPad;
    const uint16_t* in = act_buf[cur];
    uint16_t* outb = act_buf[cur ^ 1];
    const bool last = (l == a.sh.n_layers - 1);
    const int n_tiles = (N + 31) / 32;
    for (int nt = wave; nt < n_tiles; nt += kBf16Waves) {
      const int col = nt * 32 + c;
      const bool col_ok = col < N;
      const float bv = col_ok ? from_bf16(bias[col]) : 0.f;
      floatx16 acc[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = bv;
#pragma unroll 1
      for (int k0 = 0; k0 < K; k0 += 16) {
        Pack8 wv;
        const uint16_t* wp = W + static_cast<size_t>(k0 + 8 * g) * N + col;
#pragma unroll
        for (int i = 0; i < 8; ++i) wv.h[i] = col_ok ? wp[static_cast<size_t>(i) * N] : uint16_t(0);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          if (mt < m_tiles) {
            Pack8 av;
            av.v = *reinterpret_cast<const uint4*>(in + (mt * 32 + c) * ld_in + k0 + 8 * g);
            acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.b, wv.b, acc[mt], 0, 0, 0);
          }
        }
      }
      // ---- epilogue: activation, then bf16 rows for the next layer or the final result ----
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        if (mt >= m_tiles) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          float v = acc[mt][r];
          if (act == EVO_ACT_TANH) v = tanhf(v);
          else if (act == EVO_ACT_RELU) v = fmaxf(v, 0.f);
          if (!last) {
            if (col_ok) outb[row * ld_out + col] = to_bf16(v);
          } else if (col_ok && row < B) {
            const size_t idx = (static_cast<size_t>(member) * B + row) * N + col;
            if (a.loss == LOSS_NONE) {
              a.out[idx] = v;
            } else {
              const float d = v - a.target[idx];
              loss_acc = fmaf(d, d, loss_acc);
            }
          }
        }
      }
    }
    __syncthreads();
    cur ^= 1;
    off += K * N + N;
  }
  if (a.loss == LOSS_NONE) return;
  // ---- fitness = -mean squared error: fixed butterfly per wave, waves added in order ---------
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) loss_acc += __shfl_xor(loss_acc, o, 64);
  if (lane == 0) red[wave] = loss_acc;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < kBf16Waves; ++w) t += red[w];
    const int A = a.sh.dims[a.sh.n_layers];
    a.fitness[member] = -t / (static_cast<float>(B) * static_cast<float>(A));
  }
}


// ---- streaming kernel for three-layer networks D0 -> H -> H -> A with H = 256 -----------------
// The weights are the dominant HBM stream (2 P bytes per member, used once).  Eight waves per
// member, wave w owning output columns 32 w .. 32 w + 31 of both hidden layers, so every wave
// streams its own slice of W1 and W2 (and waves 0..3 all of W3) with 16-byte loads.  A matrix
// B operand needs eight consecutive k at one column while memory is contiguous along the
// columns: the slice goes through a small wave-private LDS tile and comes back transposed with
// ds_read_b64_tr_b16.  Within each group of 16 lanes that instruction returns to lane l,
// element j, the 16-bit element (l & 3) of the 8 bytes addressed by lane (l >> 2) + 4 j; with
// lane r pointing at row (r >> 2), columns 4 (r & 3) .. +3 of the tile, lane l receives rows
// 0..3 of column l: four consecutive k for its own column.
typedef float floatx4v __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

__device__ __forceinline__ bf16x8 join_bf16(short4v lo, short4v hi) {
  union {
    short4v h[2];
    bf16x8 b;
  } u;
  u.h[0] = lo;
  u.h[1] = hi;
  return u.b;
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  Pack8 p;
  p.v = v;
  return p.b;
}

__device__ __forceinline__ float act_f(float v, int act) {
  if (act == EVO_ACT_TANH) return tanhf(v);
  // max(v, 0) on the bit pattern as a signed integer: every negative float (and -0) is a negative integer, the
  // others order like themselves; one instruction where the floating-point maximum of a matrix result needs a
  // canonicalising move first, and a NaN stays a NaN
  if (act == EVO_ACT_RELU) return __int_as_float(max(__float_as_int(v), 0));
  return v;
}

// The weight stream of one wave is a fixed sequence of B operands ("units", 1 KB each): D0/16 of
// layer 1, 16 of layer 2 and (waves 0..3) 8 of layer 3.  kDepth units are kept in flight in a
// register ring (one 16-byte load per lane and unit); the loads do not depend on activations, so
// the stream runs ahead across the layer boundaries and the workgroup barriers.
constexpr int kDepth = 12;
constexpr int kStageLd = 40;   // row stride (elements) of the 16 x 32 staging tile of layers 1, 2
constexpr int kStageLd3 = 24;  // row stride of the 32 x 16 staging tile of layer 3
constexpr int kStageElems = 32 * kStageLd3;  // 768 elements >= 16 * kStageLd

// At most 64 observations per member (one tile); more go to the register-resident kernel below.
// RELU: the hidden activations are ReLU and the output is linear (the shape's usual policy), which
// removes the per-value activation switch from the epilogues.
template <int D0, int H, int A, bool RELU>
__global__ __launch_bounds__(512, 4) void mlp_bf16_stream_kernel(Bf16Args a) {
  static_assert(H == 256 && D0 % 32 == 0 && A == 16, "shape of the streaming kernel");
  constexpr int LD0 = D0 + kRowPad, LDH = H + kRowPad;
  constexpr int U1 = D0 / 16, U2 = H / 16, U3 = H / 32, UT = U1 + U2 + U3;
  __shared__ __attribute__((aligned(16))) uint16_t x_s[64 * LD0];
  __shared__ __attribute__((aligned(16))) uint16_t h_s[64 * LDH];
  __shared__ __attribute__((aligned(16))) uint16_t stage_s[8 * kStageElems];
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 31, g = lane >> 5;
  const int c16 = lane & 15, g4 = lane >> 4;
  uint16_t* stage = stage_s + wave * kStageElems;
  const int member = blockIdx.x, B = a.B;
  const uint16_t* theta = a.params + static_cast<size_t>(member) * a.sh.P;
  const uint16_t* W1 = theta;
  const uint16_t* B1 = W1 + D0 * H;
  const uint16_t* W2 = B1 + H;
  const uint16_t* B2 = W2 + H * H;
  const uint16_t* W3 = B2 + H;
  const uint16_t* B3 = W3 + H * A;
  const bool tail = wave < 4;  // waves that also run layer 3

  u32x4v ring[kDepth];
  // unit u -> its 16-byte load (compile-time u after unrolling).  Layers 1, 2: tile of 16 rows x
  // 32 columns, lane = (row lane >> 2, 8 columns from 8 (lane & 3)); layer 3: 32 rows x 16 columns,
  // lane = (row lane >> 1, 8 columns from 8 (lane & 1)).
  const uint16_t* p12 = theta + static_cast<size_t>(lane >> 2) * H + 32 * wave + 8 * (lane & 3);
  const uint16_t* p3 = W3 + (lane >> 1) * A + 8 * (lane & 1);
  auto issue = [&](int u) {
    u32x4v& r = ring[u % kDepth];
    if (u < U1) r = *reinterpret_cast<const u32x4v*>(p12 + static_cast<size_t>(16 * u) * H);
    else if (u < U1 + U2) r = *reinterpret_cast<const u32x4v*>(p12 + (W2 - theta) + static_cast<size_t>(16 * (u - U1)) * H);
    else if (u < UT && tail) r = *reinterpret_cast<const u32x4v*>(p3 + 32 * (u - U1 - U2) * A);
  };
  // registers of unit u -> staging tile -> transposed B operand of this lane
  auto operand12 = [&](int u) -> bf16x8 {
    *reinterpret_cast<u32x4v*>(stage + (lane >> 2) * kStageLd + 8 * (lane & 3)) = ring[u % kDepth];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint16_t* q = stage + (8 * g + (c16 >> 2)) * kStageLd + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return join_bf16(lo, hi);
  };
  auto operand3 = [&](int u) -> bf16x8 {
    *reinterpret_cast<u32x4v*>(stage + (lane >> 1) * kStageLd3 + 8 * (lane & 1)) = ring[u % kDepth];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint16_t* q = stage + (8 * g4 + (c16 >> 2)) * kStageLd3 + 4 * (lane & 3);
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd3));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return join_bf16(lo, hi);
  };
  // rows = observations 8 rr + 4 g + i, columns = the wave's neurons 32 wave + c; the two column biases are
  // fetched here, ahead of the tile (a load at the point of use would sit between two layers)
  const float bias_col[2] = {from_bf16(B1[32 * wave + c]), from_bf16(B2[32 * wave + c])};
  auto bias_rows = [&](int layer, floatx16 (&acc)[2]) {
    const float b = bias_col[layer];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][r] = b;
  };
  auto store_rows = [&](const floatx16 (&acc)[2], int act) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        h_s[row * LDH + 32 * wave + c] = to_bf16(act_f(acc[mt][r], act));
      }
  };
  const float bias3 = from_bf16(B3[c16]);  // layer 3: column = output c16
  float loss_acc = 0.f;
  // the observation loads go first so that waiting for them does not drain the weight stream
  constexpr int kObsPieces = 64 * D0 / 4 / 512;
  float4 ov[kObsPieces];
  {
    const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;
#pragma unroll
    for (int j = 0; j < kObsPieces; ++j) {
      const int i = tid + 512 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      ov[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < B) ov[j] = reinterpret_cast<const float4*>(obs + static_cast<size_t>(r) * D0)[d4];
    }
  }
#pragma unroll
  for (int u = 0; u < kDepth; ++u) issue(u);

  // ---- observations -> bf16 rows (rows beyond B are zero) ---------------------------------------
#pragma unroll
  for (int j = 0; j < kObsPieces; ++j) {
    const int i = tid + 512 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
    uint2 pk;
    pk.x = pack_bf16x2(ov[j].x, ov[j].y);
    pk.y = pack_bf16x2(ov[j].z, ov[j].w);
    *reinterpret_cast<uint2*>(x_s + r * LD0 + 4 * d4) = pk;
  }
  // targets of this lane's four output rows (layer 3 tile of wave < 4): output c16 of observations 16 wave + 4 g4 + i
  float tgt[4] = {0.f, 0.f, 0.f, 0.f};
  if (tail && a.loss != LOSS_NONE) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 16 * wave + 4 * g4 + i;
      if (row < B) tgt[i] = a.target[(static_cast<size_t>(member) * B + row) * A + c16];
    }
  }
  __syncthreads();

  // ---- layer 1 ----------------------------------------------------------------------------------
  floatx16 acc[2];
  bias_rows(0, acc);
#pragma unroll
  for (int u = 0; u < U1; ++u) {
    const bf16x8 bv = operand12(u);
    issue(u + kDepth);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const uint4 av = *reinterpret_cast<const uint4*>(x_s + (mt * 32 + c) * LD0 + 16 * u + 8 * g);
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), bv, acc[mt], 0, 0, 0);
    }
  }
  store_rows(acc, RELU ? EVO_ACT_RELU : a.sh.act[0]);
  __syncthreads();

  // ---- layer 2 ----------------------------------------------------------------------------------
  bias_rows(1, acc);
#pragma unroll
  for (int u = U1; u < U1 + U2; ++u) {
    const bf16x8 bv = operand12(u);
    issue(u + kDepth);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const uint4 av = *reinterpret_cast<const uint4*>(h_s + (mt * 32 + c) * LDH + 16 * (u - U1) + 8 * g);
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), bv, acc[mt], 0, 0, 0);
    }
  }
  __syncthreads();  // every wave has read h1: the buffer can take h2
  store_rows(acc, RELU ? EVO_ACT_RELU : a.sh.act[1]);
  __syncthreads();

  // ---- layer 3: four waves, one 16-row tile each (16x16x32 tiles: lane = 16 g4 + c16) -------------
  if (tail) {
    floatx4v o = {bias3, bias3, bias3, bias3};
#pragma unroll
    for (int u = U1 + U2; u < UT; ++u) {
      const bf16x8 bv = operand3(u);
      issue(u + kDepth);
      const uint4 av = *reinterpret_cast<const uint4*>(h_s + (16 * wave + c16) * LDH + 32 * (u - U1 - U2) + 8 * g4);
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), bv, o, 0, 0, 0);
    }
    const int act = RELU ? EVO_ACT_NONE : a.sh.act[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 16 * wave + 4 * g4 + i;
      const float v = act_f(o[i], act);
      if (row < B) {
        if (a.loss == LOSS_NONE) {
          a.out[(static_cast<size_t>(member) * B + row) * A + c16] = v;
        } else {
          const float d = v - tgt[i];
          loss_acc = fmaf(d, d, loss_acc);
        }
      }
    }
  }
  if (a.loss == LOSS_NONE) return;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) loss_acc += __shfl_xor(loss_acc, o, 64);
  if (lane == 0 && tail) red[wave] = loss_acc;
  __syncthreads();
  if (tid == 0) a.fitness[member] = -(red[0] + red[1] + red[2] + red[3]) / (static_cast<float>(B) * A);
}

// ---- ask fused into the forward: one workgroup per antithetic pair, the population never written -------
// The streaming kernel above is bound by the weight stream that ask wrote a moment earlier (cfg4: 709 MB
// written and read straight back).  Here the two members of a pair are evaluated together and their weights
// are never in memory: where the streaming kernel loads the 16 bytes of unit u that belong to a lane (eight
// consecutive parameters), this kernel draws them -- mu and sigma of those eight parameters (fp32, shared by
// every pair, so they come from the L2), the two Philox blocks of the pair's noise, theta+ and theta- formed
// and rounded exactly as pgpe_ask stores them -- and hands each member's 16 bytes to the same staging tile and
// transposed read.  One draw serves both members; the matrix products, epilogues and the loss follow the
// streaming kernel instruction for instruction, so the fitness is bit for bit that of ask followed by rollout.
// The kernel is bound by the noise generation (the cost of ask alone); the forward rides along.
// The small output layer's operands are drawn once per workgroup (wave w draws rows 32 w .. 32 w + 31) and left
// in LDS in operand form for the four waves that run layer 3.
struct PairArgs {
  MlpShape sh;
  const float* mu;
  const float* sigma;
  uint32_t key0, key1, gen;
  const uint32_t* gen_dev;
  const float* obs;
  int64_t obs_stride;
  int B;
  float* out;
  const float* target;
  float* fitness;
  int loss;
};

// theta+ and theta- of parameter i as pgpe_ask stores them in bfloat16, widened again.
__device__ __forceinline__ void theta_pair_at(const PairArgs& a, uint32_t pair, uint32_t gen, int i, float& plus,
                                              float& minus) {
  float z[4];
  philox_normal4(static_cast<uint32_t>(i >> 2), pair, gen, EVO_TAG_NOISE, a.key0, a.key1, z);
  const int e = i & 3;
  const float zz = e == 0 ? z[0] : (e == 1 ? z[1] : (e == 2 ? z[2] : z[3]));
  const float m = a.mu[i], sg = a.sigma[i];
  plus = from_bf16(to_bf16(fmaf(sg, zz, m)));
  minus = from_bf16(to_bf16(fmaf(-sg, zz, m)));
}

template <int D0, int H, int A>
constexpr size_t pair_lds_bytes() {
  return (2 * 64 * (D0 + kRowPad) + 2 * 64 * (H + kRowPad) + 8 * kStageElems) * sizeof(uint16_t) +
         2 * (H / 32) * 64 * 16;
}

template <int D0, int H, int A, bool RELU>
__global__ __launch_bounds__(512) void mlp_bf16_pair_kernel(PairArgs a) {
  static_assert(H == 256 && D0 % 32 == 0 && A == 16, "shape of the pair kernel");
  constexpr int LD0 = D0 + kRowPad, LDH = H + kRowPad;
  constexpr int U1 = D0 / 16, U2 = H / 16, U3 = H / 32;
  constexpr int oB1 = D0 * H, oW2 = oB1 + H, oB2 = oW2 + H * H, oW3 = oB2 + H, oB3 = oW3 + H * A;
  static_assert(U3 == 8, "one output-layer unit per wave");
  extern __shared__ __attribute__((aligned(16))) uint16_t pair_lds[];
  uint16_t* x_s = pair_lds;                         // [2][64][LD0]
  uint16_t* h_s = x_s + 2 * 64 * LD0;               // [2][64][LDH]
  uint16_t* stage_s = h_s + 2 * 64 * LDH;           // [8][kStageElems]
  u32x4v* w3_s = reinterpret_cast<u32x4v*>(stage_s + 8 * kStageElems);  // [2][U3][64] output-layer operands
  __shared__ float red[2][4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 31, g = lane >> 5;
  const int c16 = lane & 15, g4 = lane >> 4;
  uint16_t* stage = stage_s + wave * kStageElems;
  const uint32_t pair = blockIdx.x;
  const uint32_t gen = a.gen_dev ? *a.gen_dev : a.gen;
  const int B = a.B;
  const bool tail = wave < 4;  // waves that also run layer 3

  // ---- the draw of unit u: mu and sigma of the lane's eight parameters, fetched kAhead units early ------
  constexpr int kAhead = 2;
  float4 ms[kAhead][4];
  const int lane12 = (lane >> 2) * H + 32 * wave + 8 * (lane & 3);  // this lane's eight parameters inside a unit
  auto unit_index = [&](int u) -> int {
    if (u < U1) return 16 * u * H + lane12;
    return oW2 + 16 * (u - U1) * H + lane12;
  };
  auto fetch = [&](int u) {
    if (u >= U1 + U2) return;
    const int i = unit_index(u);
    float4* r = ms[u % kAhead];
    r[0] = *reinterpret_cast<const float4*>(a.mu + i);
    r[1] = *reinterpret_cast<const float4*>(a.mu + i + 4);
    r[2] = *reinterpret_cast<const float4*>(a.sigma + i);
    r[3] = *reinterpret_cast<const float4*>(a.sigma + i + 4);
  };
  // eight parameters from index i (a multiple of 8): both members' 16 bytes, as pgpe_ask stores them
  auto draw8 = [&](int i, const float4 (&r)[4], u32x4v& plus, u32x4v& minus) {
    const float mu8[8] = {r[0].x, r[0].y, r[0].z, r[0].w, r[1].x, r[1].y, r[1].z, r[1].w};
    const float sg8[8] = {r[2].x, r[2].y, r[2].z, r[2].w, r[3].x, r[3].y, r[3].z, r[3].w};
    float z[8];
    philox_normal4(static_cast<uint32_t>(i >> 2), pair, gen, EVO_TAG_NOISE, a.key0, a.key1, z);
    philox_normal4(static_cast<uint32_t>(i >> 2) + 1u, pair, gen, EVO_TAG_NOISE, a.key0, a.key1, z + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      plus[e] = pack_bf16x2(fmaf(sg8[2 * e], z[2 * e], mu8[2 * e]), fmaf(sg8[2 * e + 1], z[2 * e + 1], mu8[2 * e + 1]));
      minus[e] = pack_bf16x2(fmaf(-sg8[2 * e], z[2 * e], mu8[2 * e]), fmaf(-sg8[2 * e + 1], z[2 * e + 1], mu8[2 * e + 1]));
    }
  };
  // 16 bytes of a lane -> staging tile -> transposed B operand of this lane (layers 1, 2: 16 rows x 32 columns)
  auto operand12 = [&](const u32x4v& v) -> bf16x8 {
    *reinterpret_cast<u32x4v*>(stage + (lane >> 2) * kStageLd + 8 * (lane & 3)) = v;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint16_t* q = stage + (8 * g + (c16 >> 2)) * kStageLd + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return join_bf16(lo, hi);
  };
  // layer 3: 32 rows x 16 columns
  auto operand3 = [&](const u32x4v& v) -> bf16x8 {
    *reinterpret_cast<u32x4v*>(stage + (lane >> 1) * kStageLd3 + 8 * (lane & 1)) = v;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint16_t* q = stage + (8 * g4 + (c16 >> 2)) * kStageLd3 + 4 * (lane & 3);
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd3));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return join_bf16(lo, hi);
  };

  // ---- observations and targets of both members (requested first: they come from HBM) --------------------
  constexpr int kObsPieces = 64 * D0 / 4 / 512;
  float4 ov[2][kObsPieces];
#pragma unroll
  for (int mem = 0; mem < 2; ++mem) {
    const float* obs = a.obs + static_cast<size_t>(2 * pair + mem) * a.obs_stride;
#pragma unroll
    for (int j = 0; j < kObsPieces; ++j) {
      const int i = tid + 512 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      ov[mem][j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < B) ov[mem][j] = reinterpret_cast<const float4*>(obs + static_cast<size_t>(r) * D0)[d4];
    }
  }
  fetch(0);
  fetch(1);
  float tgt[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  if (tail && a.loss != LOSS_NONE) {
#pragma unroll
    for (int mem = 0; mem < 2; ++mem)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 16 * wave + 4 * g4 + i;
        if (row < B) tgt[mem][i] = a.target[(static_cast<size_t>(2 * pair + mem) * B + row) * A + c16];
      }
  }
  // ---- output layer: wave w draws rows 32 w .. 32 w + 31 of W3 and leaves both members' operands in LDS ----
  {
    const int i = oW3 + (32 * wave + (lane >> 1)) * A + 8 * (lane & 1);
    float4 r[4];
    r[0] = *reinterpret_cast<const float4*>(a.mu + i);
    r[1] = *reinterpret_cast<const float4*>(a.mu + i + 4);
    r[2] = *reinterpret_cast<const float4*>(a.sigma + i);
    r[3] = *reinterpret_cast<const float4*>(a.sigma + i + 4);
    u32x4v plus, minus;
    draw8(i, r, plus, minus);
    w3_s[(0 * U3 + wave) * 64 + lane] = __builtin_bit_cast(u32x4v, operand3(plus));
    w3_s[(1 * U3 + wave) * 64 + lane] = __builtin_bit_cast(u32x4v, operand3(minus));
  }
  // biases of this lane's columns (layers 1, 2) and output (layer 3), both members
  float bias_col[2][2], bias3[2];
  theta_pair_at(a, pair, gen, oB1 + 32 * wave + c, bias_col[0][0], bias_col[1][0]);
  theta_pair_at(a, pair, gen, oB2 + 32 * wave + c, bias_col[0][1], bias_col[1][1]);
  theta_pair_at(a, pair, gen, oB3 + c16, bias3[0], bias3[1]);

  // ---- observations -> bf16 rows (rows beyond B are zero) ---------------------------------------
#pragma unroll
  for (int mem = 0; mem < 2; ++mem)
#pragma unroll
    for (int j = 0; j < kObsPieces; ++j) {
      const int i = tid + 512 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      uint2 pk;
      pk.x = pack_bf16x2(ov[mem][j].x, ov[mem][j].y);
      pk.y = pack_bf16x2(ov[mem][j].z, ov[mem][j].w);
      *reinterpret_cast<uint2*>(x_s + mem * 64 * LD0 + r * LD0 + 4 * d4) = pk;
    }
  __syncthreads();

  floatx16 acc[2][2];  // [member][row tile]
  auto bias_rows = [&](int layer) {
#pragma unroll
    for (int mem = 0; mem < 2; ++mem)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mem][mt][r] = bias_col[mem][layer];
  };
  auto store_rows = [&](int act) {
#pragma unroll
    for (int mem = 0; mem < 2; ++mem)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          h_s[mem * 64 * LDH + row * LDH + 32 * wave + c] = to_bf16(act_f(acc[mem][mt][r], act));
        }
  };
  // one unit of layer 1 or 2: draw, then both members' products
  auto unit = [&](int u, const uint16_t* in, int ld, int k0) {
    u32x4v pm[2];
    draw8(unit_index(u), ms[u % kAhead], pm[0], pm[1]);
    fetch(u + kAhead);
#pragma unroll
    for (int mem = 0; mem < 2; ++mem) {
      const bf16x8 bv = operand12(pm[mem]);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const uint4 av = *reinterpret_cast<const uint4*>(in + mem * 64 * ld + (mt * 32 + c) * ld + k0 + 8 * g);
        acc[mem][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), bv, acc[mem][mt], 0, 0, 0);
      }
    }
  };

  // ---- layer 1 ----------------------------------------------------------------------------------
  bias_rows(0);
#pragma unroll
  for (int u = 0; u < U1; ++u) unit(u, x_s, LD0, 16 * u);
  store_rows(RELU ? EVO_ACT_RELU : a.sh.act[0]);
  __syncthreads();

  // ---- layer 2 ----------------------------------------------------------------------------------
  bias_rows(1);
#pragma unroll
  for (int u = U1; u < U1 + U2; ++u) unit(u, h_s, LDH, 16 * (u - U1));
  __syncthreads();  // every wave has read h1: the buffer can take h2
  store_rows(RELU ? EVO_ACT_RELU : a.sh.act[1]);
  __syncthreads();

  // ---- layer 3: four waves, one 16-row tile each per member ------------------------------------------
  float loss_acc[2] = {0.f, 0.f};
  if (tail) {
#pragma unroll
    for (int mem = 0; mem < 2; ++mem) {
      floatx4v o = {bias3[mem], bias3[mem], bias3[mem], bias3[mem]};
#pragma unroll
      for (int u = 0; u < U3; ++u) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, w3_s[(mem * U3 + u) * 64 + lane]);
        const uint4 av = *reinterpret_cast<const uint4*>(h_s + mem * 64 * LDH + (16 * wave + c16) * LDH + 32 * u + 8 * g4);
        o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), bv, o, 0, 0, 0);
      }
      const int act = RELU ? EVO_ACT_NONE : a.sh.act[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 16 * wave + 4 * g4 + i;
        const float v = act_f(o[i], act);
        if (row < B) {
          if (a.loss == LOSS_NONE) {
            a.out[(static_cast<size_t>(2 * pair + mem) * B + row) * A + c16] = v;
          } else {
            const float d = v - tgt[mem][i];
            loss_acc[mem] = fmaf(d, d, loss_acc[mem]);
          }
        }
      }
    }
  }
  if (a.loss == LOSS_NONE) return;
#pragma unroll
  for (int mem = 0; mem < 2; ++mem) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) loss_acc[mem] += __shfl_xor(loss_acc[mem], o, 64);
    if (lane == 0 && tail) red[mem][wave] = loss_acc[mem];
  }
  __syncthreads();
  if (tid < 2)
    a.fitness[2 * pair + tid] = -(red[tid][0] + red[tid][1] + red[tid][2] + red[tid][3]) / (static_cast<float>(B) * A);
}

// Two floats rounded to bf16 (one conversion instruction) and max(x, 0) taken on both halves at once.
typedef short short2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t relu_pack_bf16x2(float lo, float hi) {
  const bf16x2_t r = __builtin_convertvector(float2v{lo, hi}, bf16x2_t);
  const short2v h = __builtin_elementwise_max(__builtin_bit_cast(short2v, r), short2v{0, 0});
  return __builtin_bit_cast(uint32_t, h);
}

// ---- register-resident kernel for more than 64 observations per member -----------------------------
// With hundreds of observations per member the weights are a small part of the traffic and the layer
// products are real matrix work.  Four waves per member; wave w owns neurons 64 w .. 64 w + 63 of both
// hidden layers, i.e. two 32-neuron tiles, and builds every matrix operand of its weights once (a
// prologue: 16-byte loads, the wave-private staging tile and the transposed read of the streaming
// kernel), 48 operands = 192 registers per lane, the member's 173 KB across the workgroup.  The tile
// loop over 64 observations then runs with no weight traffic at all.  Products are transposed (rows =
// neurons, columns = 32 observations): one 16-byte LDS read of activations feeds two matrix
// instructions (the wave's two neuron tiles), which halves the LDS traffic per instruction against
// one tile per wave -- with one tile per wave the 1 KB operand per instruction is exactly the CU's
// LDS bandwidth when all four SIMDs issue back to back.  The observations of the next tile are
// requested before the current tile's layers run.
template <int D0, int H, int A, int MT, bool RELU>
__global__ __launch_bounds__(256) void mlp_bf16_resident_kernel(Bf16Args a) {
  constexpr int kRows = 32 * MT;  // observations per pass of the tile loop
  static_assert(H == 256 && D0 % 32 == 0 && A == 16 && (MT == 2 || MT == 4), "shape of the resident kernel");
  constexpr int LD0 = D0 + kRowPad, LDH = H + kRowPad;
  constexpr int U1 = D0 / 16, U2 = H / 16, U3 = H / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t resident_lds[];  // resident_lds_bytes(MT)
  uint16_t* x_s = resident_lds;                  // [kRows][LD0]
  uint16_t* h_s = x_s + kRows * LD0;             // [kRows][LDH]
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 31, g = lane >> 5;
  const int c16 = lane & 15, g4 = lane >> 4;
  const int member = blockIdx.x, B = a.B;
  const uint16_t* theta = a.params + static_cast<size_t>(member) * a.sh.P;
  const uint16_t* W1 = theta;
  const uint16_t* B1 = W1 + D0 * H;
  const uint16_t* W2 = B1 + H;
  const uint16_t* B2 = W2 + H * H;
  const uint16_t* W3 = B2 + H;
  const uint16_t* B3 = W3 + H * A;

  // observations of a tile: 64 x D0 floats, 16-byte pieces, kObsPieces per thread
  constexpr int kObsPieces = kRows * D0 / 4 / 256;
  const float* obs_member = a.obs + static_cast<size_t>(member) * a.obs_stride;
  float4 ov[kObsPieces];
  auto load_obs = [&](int row0) {
#pragma unroll
    for (int j = 0; j < kObsPieces; ++j) {
      const int i = tid + 256 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      ov[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row0 + r < B) ov[j] = reinterpret_cast<const float4*>(obs_member + static_cast<size_t>(row0 + r) * D0)[d4];
    }
  };
  load_obs(0);

  // ---- prologue: this wave's matrix operands ---------------------------------------------------------
  // 16-byte loads of W (contiguous along the columns), a wave-private staging tile in LDS, and the
  // transposed read that hands every lane eight consecutive k of its column.  Four tiles per round trip
  // through LDS; the staging tiles borrow the wave's quarter of the (still unused) hidden-activation buffer.
  constexpr int kBatch = 4;
  uint16_t* stage = h_s + wave * (kRows * LDH / 4);
  static_assert(kBatch * kStageElems <= kRows * LDH / 4, "staging tiles fit into a quarter of the activation buffer");
  auto fence_wave = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  // 16 rows x 32 columns of W1 / W2 per tile
  auto transposed12 = [&](const u32x4v* raw, bf16x8* out) {
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      *reinterpret_cast<u32x4v*>(stage + j * kStageElems + (lane >> 2) * kStageLd + 8 * (lane & 3)) = raw[j];
    fence_wave();
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const uint16_t* q = stage + j * kStageElems + (8 * g + (c16 >> 2)) * kStageLd + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
      const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd));
      out[j] = join_bf16(lo, hi);
    }
    fence_wave();
  };
  // 32 rows x 16 columns of W3 per tile
  auto transposed3 = [&](const u32x4v* raw, bf16x8* out) {
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      *reinterpret_cast<u32x4v*>(stage + j * kStageElems + (lane >> 1) * kStageLd3 + 8 * (lane & 1)) = raw[j];
    fence_wave();
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const uint16_t* q = stage + j * kStageElems + (8 * g4 + (c16 >> 2)) * kStageLd3 + 4 * (lane & 3);
      const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q));
      const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(q + 4 * kStageLd3));
      out[j] = join_bf16(lo, hi);
    }
    fence_wave();
  };
  static_assert(U1 % kBatch == 0 && U2 % kBatch == 0 && U3 % kBatch == 0, "operands come in rounds of four");
  bf16x8 w1[2][U1], w2[2][U2], w3[U3];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint16_t* p12 = theta + static_cast<size_t>(lane >> 2) * H + 32 * (2 * wave + t) + 8 * (lane & 3);
    u32x4v raw[U1 + U2];
#pragma unroll
    for (int u = 0; u < U1; ++u) raw[u] = *reinterpret_cast<const u32x4v*>(p12 + static_cast<size_t>(16 * u) * H);
#pragma unroll
    for (int u = 0; u < U2; ++u)
      raw[U1 + u] = *reinterpret_cast<const u32x4v*>(p12 + (W2 - theta) + static_cast<size_t>(16 * u) * H);
#pragma unroll
    for (int u = 0; u < U1; u += kBatch) transposed12(raw + u, w1[t] + u);
#pragma unroll
    for (int u = 0; u < U2; u += kBatch) transposed12(raw + U1 + u, w2[t] + u);
  }
  {
    const uint16_t* p3 = W3 + (lane >> 1) * A + 8 * (lane & 1);
    u32x4v raw[U3];
#pragma unroll
    for (int u = 0; u < U3; ++u) raw[u] = *reinterpret_cast<const u32x4v*>(p3 + 32 * u * A);
#pragma unroll
    for (int u = 0; u < U3; u += kBatch) transposed3(raw + u, w3 + u);
  }
  // The hidden layers' biases enter as one more product: a weight operand whose k = 0 column is the bias
  // of the lane's neuron (everything else zero) times an activation operand whose k = 0 row is one.  The
  // accumulators then start from that product with a zero addend: no bias registers, no initial copies.
  bf16x8 wb1[2], wb2[2], ones;
  {
    Pack8 p;
    p.v = make_uint4(0u, 0u, 0u, 0u);
    if (g == 0) p.h[0] = 0x3F80;  // bf16 1.0
    ones = p.b;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      p.v = make_uint4(0u, 0u, 0u, 0u);
      if (g == 0) p.h[0] = B1[64 * wave + 32 * t + c];
      wb1[t] = p.b;
      p.v = make_uint4(0u, 0u, 0u, 0u);
      if (g == 0) p.h[0] = B2[64 * wave + 32 * t + c];
      wb2[t] = p.b;
    }
  }
  float bias3[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bias3[i] = from_bf16(B3[4 * g4 + i]);

  // activation, two bf16 per word, four consecutive neurons of one observation per 8-byte store.
  // RELU: rounding keeps the sign, so max(x, 0) is taken after the rounding, on both halves of a word at
  // once as a signed 16-bit maximum (a negative bf16 is a negative int16).
  auto store_rows = [&](const floatx16& acc, int t, int mt, int act) {
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      uint2 pk;
      if (RELU) {
        pk.x = relu_pack_bf16x2(acc[4 * rr], acc[4 * rr + 1]);
        pk.y = relu_pack_bf16x2(acc[4 * rr + 2], acc[4 * rr + 3]);
      } else {
        pk.x = pack_bf16x2(act_f(acc[4 * rr], act), act_f(acc[4 * rr + 1], act));
        pk.y = pack_bf16x2(act_f(acc[4 * rr + 2], act), act_f(acc[4 * rr + 3], act));
      }
      *reinterpret_cast<uint2*>(h_s + (mt * 32 + c) * LDH + 64 * wave + 32 * t + 8 * rr + 4 * g) = pk;
    }
  };
  // One layer's products: step s = (k-slice s / 2, observation tile s % 2) reads one activation operand and
  // feeds the wave's two neuron tiles.  The reads run kAhead steps ahead of the matrix instructions; the
  // scheduling fences keep that order (left alone, the compiler issues each read right before its use).
  constexpr int kAhead = 3;
  auto layer_products = [&](floatx16 (&acc)[2][MT], const uint16_t* in, int ld, const bf16x8 (&wb)[2], auto wt,
                            auto steps_c) {
    constexpr int kSteps = decltype(steps_c)::value;
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc[0][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[0], ones, zero, 0, 0, 0);
      acc[1][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[1], ones, zero, 0, 0, 0);
    }
    uint4 av[kSteps];
    auto read = [&](int s) { av[s] = *reinterpret_cast<const uint4*>(in + ((s % MT) * 32 + c) * ld + 16 * (s / MT) + 8 * g); };
#pragma unroll
    for (int s = 0; s < kAhead && s < kSteps; ++s) read(s);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      if (s + kAhead < kSteps) read(s + kAhead);
      __builtin_amdgcn_sched_barrier(0);
      acc[0][s % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wt(0, s / MT), as_bf16x8(av[s]), acc[0][s % MT], 0, 0, 0);
      acc[1][s % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wt(1, s / MT), as_bf16x8(av[s]), acc[1][s % MT], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  float loss_acc = 0.f;
#pragma unroll 1
  for (int row0 = 0; row0 < B; row0 += kRows) {
    // ---- observations -> bf16 rows (rows beyond B are zero); the next tile's are requested at once ----
#pragma unroll
    for (int j = 0; j < kObsPieces; ++j) {
      const int i = tid + 256 * j, r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      uint2 pk;
      pk.x = pack_bf16x2(ov[j].x, ov[j].y);
      pk.y = pack_bf16x2(ov[j].z, ov[j].w);
      *reinterpret_cast<uint2*>(x_s + r * LD0 + 4 * d4) = pk;
    }
    if (row0 + kRows < B) load_obs(row0 + kRows);
    // layer 3: a wave takes MT / 2 groups of 16 observations; lane = observation c16 of a group, outputs 4 g4 ..
    constexpr int kGroups = MT / 2;
    float4 tgt[kGroups];
#pragma unroll
    for (int gi = 0; gi < kGroups; ++gi) {
      const int row = row0 + 16 * (kGroups * wave + gi) + c16;
      tgt[gi] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (a.loss != LOSS_NONE && row < B)
        tgt[gi] = *reinterpret_cast<const float4*>(a.target + (static_cast<size_t>(member) * B + row) * A + 4 * g4);
    }
    __syncthreads();  // x_s is complete; every wave has left layer 3 of the previous tile

    // ---- layer 1 ------------------------------------------------------------------------------------
    floatx16 acc[2][MT];
    layer_products(acc, x_s, LD0, wb1, [&](int t, int u) { return w1[t][u]; }, std::integral_constant<int, MT * U1>{});
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) store_rows(acc[t][mt], t, mt, RELU ? EVO_ACT_RELU : a.sh.act[0]);
    __syncthreads();

    // ---- layer 2 ------------------------------------------------------------------------------------
    layer_products(acc, h_s, LDH, wb2, [&](int t, int u) { return w2[t][u]; }, std::integral_constant<int, MT * U2>{});
    __syncthreads();  // every wave has read h1: the buffer can take h2
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) store_rows(acc[t][mt], t, mt, RELU ? EVO_ACT_RELU : a.sh.act[1]);
    __syncthreads();

    // ---- layer 3: 16x16x32 tiles (lane = 16 g4 + c16), MT / 2 groups of 16 observations per wave ----------
#pragma unroll
    for (int gi = 0; gi < kGroups; ++gi) {
      const int local = 16 * (kGroups * wave + gi) + c16, row = row0 + local;
      floatx4v o = {bias3[0], bias3[1], bias3[2], bias3[3]};
#pragma unroll
      for (int u = 0; u < U3; ++u) {
        const uint4 av = *reinterpret_cast<const uint4*>(h_s + local * LDH + 32 * u + 8 * g4);
        o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3[u], as_bf16x8(av), o, 0, 0, 0);
      }
      if (row < B) {
        const int act = RELU ? EVO_ACT_NONE : a.sh.act[2];
        const float v0 = act_f(o[0], act), v1 = act_f(o[1], act), v2 = act_f(o[2], act), v3 = act_f(o[3], act);
        if (a.loss == LOSS_NONE) {
          *reinterpret_cast<float4*>(a.out + (static_cast<size_t>(member) * B + row) * A + 4 * g4) = make_float4(v0, v1, v2, v3);
        } else {
          const float d0 = v0 - tgt[gi].x, d1 = v1 - tgt[gi].y, d2 = v2 - tgt[gi].z, d3 = v3 - tgt[gi].w;
          loss_acc = fmaf(d0, d0, loss_acc);
          loss_acc = fmaf(d1, d1, loss_acc);
          loss_acc = fmaf(d2, d2, loss_acc);
          loss_acc = fmaf(d3, d3, loss_acc);
        }
      }
    }
  }
  if (a.loss == LOSS_NONE) return;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) loss_acc += __shfl_xor(loss_acc, o, 64);
  if (lane == 0) red[wave] = loss_acc;
  __syncthreads();
  if (tid == 0) a.fitness[member] = -(red[0] + red[1] + red[2] + red[3]) / (static_cast<float>(B) * A);
}

template <int D0, int H, int MT>
constexpr size_t resident_lds_bytes() {
  return static_cast<size_t>(32 * MT) * (D0 + kRowPad + H + kRowPad) * sizeof(uint16_t);
}

constexpr int kStreamMaxRows = 4096;  // observations per member of the streaming kernel (tiles of 64)

static bool stream_shape(const MlpShape& sh, int B) {
  return sh.n_layers == 3 && sh.dims[0] == 64 && sh.dims[1] == 256 && sh.dims[2] == 256 && sh.dims[3] == 16 &&
         B <= kStreamMaxRows;
}

int mlp_bf16_supported(const MlpShape& sh, int B) {
  if (B >= 1 && stream_shape(sh, B)) return EVO_OK;  // the streaming kernel walks over tiles of 64 rows
  EVO_REQUIRE(B >= 1 && B <= kMaxRows, EVO_ERR_UNSUPPORTED, "bf16 MLP: B must be in [1, %d] (got %d)", kMaxRows, B);
  EVO_REQUIRE(sh.max_width <= kMaxWidth, EVO_ERR_UNSUPPORTED, "bf16 MLP: widths above %d are not supported (%d)",
              kMaxWidth, sh.max_width);
  for (int l = 0; l < sh.n_layers; ++l)
    EVO_REQUIRE(sh.dims[l] % 16 == 0, EVO_ERR_UNSUPPORTED,
                "bf16 MLP: every layer input width must be a multiple of 16 (dims[%d] = %d)", l, sh.dims[l]);
  return EVO_OK;
}

int launch_mlp_bf16(const MlpShape& sh, const uint16_t* params, const float* obs, int64_t obs_stride, int pop, int B,
                    float* out, int loss, const void* target, float* fitness, hipStream_t s) {
  EVO_REQUIRE(loss != LOSS_CE, EVO_ERR_UNSUPPORTED, "bf16 MLP: the classification loss is not implemented");
  Bf16Args a;
  a.sh = sh, a.params = params, a.obs = obs, a.obs_stride = obs_stride, a.B = B;
  a.out = out, a.target = static_cast<const float*>(target), a.fitness = fitness, a.loss = loss;
  if (stream_shape(sh, B)) {
    a.buf_elems = 0;
    const bool relu = sh.act[0] == EVO_ACT_RELU && sh.act[1] == EVO_ACT_RELU && sh.act[2] == EVO_ACT_NONE;
    if (B <= 64) {
      if (relu)
        hipLaunchKernelGGL((mlp_bf16_stream_kernel<64, 256, 16, true>), dim3(pop), dim3(512), 0, s, a);
      else
        hipLaunchKernelGGL((mlp_bf16_stream_kernel<64, 256, 16, false>), dim3(pop), dim3(512), 0, s, a);
    } else {
      constexpr int MT = 2;  // 64 observations per pass (128 measured slower: 2.17 vs 1.64 ms at B = 2048)
      constexpr size_t lds = resident_lds_bytes<64, 256, MT>();
      const void* fn = relu ? reinterpret_cast<const void*>(&mlp_bf16_resident_kernel<64, 256, 16, MT, true>)
                            : reinterpret_cast<const void*>(&mlp_bf16_resident_kernel<64, 256, 16, MT, false>);
      hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
      EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
      if (relu)
        hipLaunchKernelGGL((mlp_bf16_resident_kernel<64, 256, 16, MT, true>), dim3(pop), dim3(256), lds, s, a);
      else
        hipLaunchKernelGGL((mlp_bf16_resident_kernel<64, 256, 16, MT, false>), dim3(pop), dim3(256), lds, s, a);
      return check_launch("mlp_bf16_resident_kernel");
    }
    return check_launch("mlp_bf16_stream_kernel");
  }
  const int rows = ((B + 31) / 32) * 32;
  a.buf_elems = rows * (sh.max_width + kRowPad);
  const size_t shmem = static_cast<size_t>(a.buf_elems) * 2 * sizeof(uint16_t);
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
    EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL(mlp_bf16_kernel, dim3(pop), dim3(kBf16Threads), shmem, s, a);
  return check_launch("mlp_bf16_kernel");
}

int mlp_bf16_pair_supported(const MlpShape& sh, int B) {
  EVO_REQUIRE(stream_shape(sh, B) && B <= 64, EVO_ERR_UNSUPPORTED,
              "ask fused with the forward: the policy must be the bfloat16 MLP 64-256-256-16 with at most 64 "
              "observations per member");
  return EVO_OK;
}

int launch_mlp_bf16_pair(const MlpShape& sh, const float* mu, const float* sigma, uint64_t seed, uint32_t gen,
                         const uint32_t* gen_dev, const float* obs, int64_t obs_stride, int pop, int B, float* out,
                         int loss, const void* target, float* fitness, hipStream_t s) {
  EVO_REQUIRE(loss != LOSS_CE, EVO_ERR_UNSUPPORTED, "bf16 MLP: the classification loss is not implemented");
  PairArgs a;
  a.sh = sh, a.mu = mu, a.sigma = sigma;
  a.key0 = static_cast<uint32_t>(seed), a.key1 = static_cast<uint32_t>(seed >> 32), a.gen = gen, a.gen_dev = gen_dev;
  a.obs = obs, a.obs_stride = obs_stride, a.B = B;
  a.out = out, a.target = static_cast<const float*>(target), a.fitness = fitness, a.loss = loss;
  const bool relu = sh.act[0] == EVO_ACT_RELU && sh.act[1] == EVO_ACT_RELU && sh.act[2] == EVO_ACT_NONE;
  constexpr size_t lds = pair_lds_bytes<64, 256, 16>();
  static_assert(lds + 64 <= 160 * 1024, "LDS budget of a CU");
  const void* fn = relu ? reinterpret_cast<const void*>(&mlp_bf16_pair_kernel<64, 256, 16, true>)
                        : reinterpret_cast<const void*>(&mlp_bf16_pair_kernel<64, 256, 16, false>);
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (e != hipSuccess) (void)hipGetLastError();
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
  if (relu)
    hipLaunchKernelGGL((mlp_bf16_pair_kernel<64, 256, 16, true>), dim3(pop / 2), dim3(512), lds, s, a);
  else
    hipLaunchKernelGGL((mlp_bf16_pair_kernel<64, 256, 16, false>), dim3(pop / 2), dim3(512), lds, s, a);
  return check_launch("mlp_bf16_pair_kernel");
}

}  // namespace evo
