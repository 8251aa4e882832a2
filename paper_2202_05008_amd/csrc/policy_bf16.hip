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
#include "kernels.h"

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

__device__ __forceinline__ uint16_t to_bf16(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((b >> 16) | 0x0040u);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return static_cast<uint16_t>(b >> 16);
}

__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

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
#pragma unroll 2
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
// pulls its own slice of W1 and W2 straight from HBM into matrix B-operand registers: all loads
// of a layer are issued before the layer is computed (they do not depend on activations), which
// keeps tens of kilobytes in flight per CU without any staging through LDS or barriers for the
// weights.  A B operand needs eight consecutive k at one column, i.e. eight 2-byte loads with a
// row stride; 32 lanes of a row group cover 64 contiguous bytes per load.
typedef float floatx4v __attribute__((ext_vector_type(4)));

struct RawB {
  uint32_t h[8];  // eight 16-bit loads, one per k row
};

// Issue the eight row loads of one B operand: rows k, k+1, .. k+7 of column `col`.
__device__ __forceinline__ void issue_b(const uint16_t* __restrict__ W, int k, int col, int N, RawB& r) {
  const uint16_t* wp = W + static_cast<size_t>(k) * N + col;
#pragma unroll
  for (int i = 0; i < 8; ++i) r.h[i] = wp[static_cast<size_t>(i) * N];
}

__device__ __forceinline__ bf16x8 pack_b(const RawB& r) {
  Pack8 p;
  p.v = make_uint4(r.h[0] | (r.h[1] << 16), r.h[2] | (r.h[3] << 16), r.h[4] | (r.h[5] << 16), r.h[6] | (r.h[7] << 16));
  return p.b;
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  Pack8 p;
  p.v = v;
  return p.b;
}

__device__ __forceinline__ float act_f(float v, int act) {
  if (act == EVO_ACT_TANH) return tanhf(v);
  if (act == EVO_ACT_RELU) return fmaxf(v, 0.f);
  return v;
}

// The weight stream of one wave is a fixed sequence of B operands ("units"): D0/16 of layer 1,
// 16 of layer 2 and (waves 0..3) 8 of layer 3.  kDepth units are kept in flight in a register
// ring; the loads do not depend on activations, so the stream runs ahead across the layer
// boundaries and the workgroup barriers.
constexpr int kDepth = 6;

template <int D0, int H, int A>
__global__ __launch_bounds__(512, 4) void mlp_bf16_stream_kernel(Bf16Args a) {
  static_assert(H == 256 && D0 % 16 == 0 && A == 16, "shape of the streaming kernel");
  constexpr int LD0 = D0 + kRowPad, LDH = H + kRowPad;
  constexpr int U1 = D0 / 16, U2 = H / 16, U3 = H / 32, UT = U1 + U2 + U3;
  __shared__ __attribute__((aligned(16))) uint16_t x_s[64 * LD0];
  __shared__ __attribute__((aligned(16))) uint16_t h_s[64 * LDH];
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
  const int col = 32 * wave + c;
  const bool tail = wave < 4;  // waves that also run layer 3

  RawB ring[kDepth];
  // unit u -> its loads (compile-time u after unrolling)
  auto issue = [&](int u) {
    RawB& r = ring[u % kDepth];
    if (u < U1) issue_b(W1, 16 * u + 8 * g, col, H, r);
    else if (u < U1 + U2) issue_b(W2, 16 * (u - U1) + 8 * g, col, H, r);
    else if (u < UT && tail) issue_b(W3, 32 * (u - U1 - U2) + 8 * g4, c16, A, r);
  };
#pragma unroll
  for (int u = 0; u < kDepth; ++u) issue(u);
  const float bias1 = from_bf16(B1[col]), bias2 = from_bf16(B2[col]);
  const float bias3 = from_bf16(B3[c16]);

  // ---- observations -> bf16 rows (rows beyond B are zero) ---------------------------------------
  {
    const float* obs = a.obs + static_cast<size_t>(member) * a.obs_stride;
    for (int i = tid; i < 64 * D0 / 4; i += 512) {
      const int r = i / (D0 / 4), d4 = i - r * (D0 / 4);
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < B) v = reinterpret_cast<const float4*>(obs + static_cast<size_t>(r) * D0)[d4];
      uint2 pk;
      pk.x = to_bf16(v.x) | (static_cast<uint32_t>(to_bf16(v.y)) << 16);
      pk.y = to_bf16(v.z) | (static_cast<uint32_t>(to_bf16(v.w)) << 16);
      *reinterpret_cast<uint2*>(x_s + r * LD0 + 4 * d4) = pk;
    }
  }
  // targets of this lane's four output rows (layer 3 tile of wave < 4)
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
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = bias1;
#pragma unroll
  for (int u = 0; u < U1; ++u) {
    const bf16x8 bv = pack_b(ring[u % kDepth]);
    issue(u + kDepth);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const uint4 av = *reinterpret_cast<const uint4*>(x_s + (mt * 32 + c) * LD0 + 16 * u + 8 * g);
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), bv, acc[mt], 0, 0, 0);
    }
  }
  {
    const int act = a.sh.act[0];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        h_s[row * LDH + col] = to_bf16(act_f(acc[mt][r], act));
      }
  }
  __syncthreads();

  // ---- layer 2 ----------------------------------------------------------------------------------
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = bias2;
#pragma unroll
  for (int u = U1; u < U1 + U2; ++u) {
    const bf16x8 bv = pack_b(ring[u % kDepth]);
    issue(u + kDepth);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const uint4 av = *reinterpret_cast<const uint4*>(h_s + (mt * 32 + c) * LDH + 16 * (u - U1) + 8 * g);
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), bv, acc[mt], 0, 0, 0);
    }
  }
  __syncthreads();  // every wave has read h1: the buffer can take h2
  {
    const int act = a.sh.act[1];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        h_s[row * LDH + col] = to_bf16(act_f(acc[mt][r], act));
      }
  }
  __syncthreads();

  // ---- layer 3: four waves, one 16-row tile each (16x16x32 tiles: lane = 16 g4 + c16) -------------
  float loss_acc = 0.f;
  if (tail) {
    floatx4v o = {bias3, bias3, bias3, bias3};
#pragma unroll
    for (int u = U1 + U2; u < UT; ++u) {
      const bf16x8 bv = pack_b(ring[u % kDepth]);
      issue(u + kDepth);
      const uint4 av = *reinterpret_cast<const uint4*>(h_s + (16 * wave + c16) * LDH + 32 * (u - U1 - U2) + 8 * g4);
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), bv, o, 0, 0, 0);
    }
    const int act = a.sh.act[2];
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

static bool stream_shape(const MlpShape& sh, int B) {
  return sh.n_layers == 3 && sh.dims[0] == 64 && sh.dims[1] == 256 && sh.dims[2] == 256 && sh.dims[3] == 16 &&
         B <= 64;
}

int mlp_bf16_supported(const MlpShape& sh, int B) {
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
    hipLaunchKernelGGL((mlp_bf16_stream_kernel<64, 256, 16>), dim3(pop), dim3(512), 0, s, a);
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

}  // namespace evo
