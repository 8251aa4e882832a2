// Population-batched fp32 ConvNet forward with a fused cross-entropy epilogue: the image
// classifier of the paper's MNIST example (Section 3, "Supervised Learning Tasks": a
// ConvNet of ~10K parameters trained as a single-step task) evaluated for every member
// with its own weights on one shared batch (Section 2, "Global Policy").
//
// conv3x3 -> ReLU -> maxpool2 -> conv3x3 -> ReLU -> maxpool2 -> dense, c1 = 8, c2 = 16.
//
// Each wavefront runs whole images end to end out of its private slice of LDS, with no
// workgroup barrier in the loop: conv1 (K = 9) on the vector ALU, conv2 (K = 72, N = 16:
// 78% of the flops) as implicit GEMM on v_mfma_f32_16x16x4_f32, the dense layer on the
// vector ALU.  Waves of one workgroup are at different stages, so matrix and vector work
// overlap on a SIMD.  Activations never leave the chip; per image the kernel reads 3 KB
// (L2 resident, shared by all members) and writes nothing.
//
// conv2 tiling.  The 16 rows of a matrix tile are 4 pooling windows x their 4 pixels, so
// that the 4 accumulator registers of a lane (rows 4q..4q+3 of column n) are exactly one
// pooling window of output channel n: max-pooling is three v_max on registers.  The
// contraction index k = tap * 8 + channel; lane group q supplies k = 4 step + q, i.e.
// input channel 4 (step & 1) + q of tap step >> 1, read from channel-major planes in LDS
// with compile-time offsets from one per-lane base.
#include "kernels.h"

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kC1 = 8, kC2 = 16;
constexpr int kHMax = 28;
constexpr int kImgW = kHMax + 2;                     // padded image row
constexpr int kImgFloats = kImgW * kImgW;            // 900
constexpr int kA1W = kHMax / 2 + 2;                  // padded conv1-output row (16)
constexpr int kA1Plane = kA1W * kA1W + 8;            // 264: plane stride = 8 mod 32 banks
constexpr int kA1Floats = kC1 * kA1Plane;            // 2112
constexpr int kA2Floats = (kHMax / 4) * (kHMax / 4) * kC2;  // 784
constexpr int kWaveFloats = kImgFloats + kA1Floats + kA2Floats;  // 3796
constexpr int kConvWaves = 4;
constexpr int kMaxCls = 16;

struct ConvArgs {
  const float* params;
  const float* images;
  const int32_t* labels;
  float* out;
  float* partial;
  int P, H, n_cls, B, chunks, imgs_per_chunk;
};

__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__global__ __launch_bounds__(64 * kConvWaves) void convnet_kernel(ConvArgs a) {
  __shared__ float lds[kConvWaves * kWaveFloats];
  __shared__ float wave_loss[kConvWaves];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* img = lds + wave * kWaveFloats;
  float* a1 = img + kImgFloats;
  float* a2 = a1 + kA1Floats;
  const int member = blockIdx.y;
  const int H = a.H, H2 = H / 2, H4 = H / 4;
  const int n_win1 = H2 * H2;  // pooled outputs of conv1
  const int n_win2 = H4 * H4;  // pooled outputs of conv2
  const int n_feat = n_win2 * kC2;
  const int n_cls = a.n_cls;

  const float* theta = a.params + static_cast<size_t>(member) * a.P;
  const float* W1 = theta;                 // [3][3][1][8]
  const float* b1 = theta + 9 * kC1;       // [8]
  const float* W2 = b1 + kC1;              // [3][3][8][16]
  const float* b2 = W2 + 9 * kC1 * kC2;    // [16]
  const float* Wd = b2 + kC2;              // [n_feat][n_cls]
  const float* bd = Wd + n_feat * n_cls;   // [n_cls]

  // zero the padded buffers once: the borders stay zero, interiors are overwritten per image
  for (int i = lane; i < kImgFloats + kA1Floats; i += 64) img[i] = 0.f;

  // conv2 weights as matrix B operands: 18 steps, k = 4 step + q, column n
  const int n = lane & 15, q = lane >> 4;
  float w2r[18];
#pragma unroll
  for (int st = 0; st < 18; ++st) w2r[st] = W2[(4 * st + q) * kC2 + n];
  const float bias2 = b2[n];
  // conv1 weights are wave-uniform: scalar registers
  float w1r[9][kC1], bias1[kC1];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int c = 0; c < kC1; ++c) w1r[t][c] = W1[t * kC1 + c];
#pragma unroll
  for (int c = 0; c < kC1; ++c) bias1[c] = b1[c];

  const int img_begin = blockIdx.x * a.imgs_per_chunk;
  const int img_end = min(a.B, img_begin + a.imgs_per_chunk);
  float loss_sum = 0.f;

  for (int im = img_begin + wave; im < img_end; im += kConvWaves) {
    // ---- stage the image into the zero-padded buffer -------------------------------------
    const float4* src = reinterpret_cast<const float4*>(a.images + static_cast<size_t>(im) * H * H);
    const int row4 = H / 4;
    for (int i = lane; i < H * row4; i += 64) {
      const int y = i / row4, x4 = i - y * row4;
      const float4 v = src[i];
      float* d = img + (y + 1) * kImgW + 4 * x4 + 1;
      d[0] = v.x, d[1] = v.y, d[2] = v.z, d[3] = v.w;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- conv1 + ReLU + pool: lane = pooled output pixel, 8 channels each ----------------
    for (int w0 = 0; w0 < n_win1; w0 += 64) {
      const int w = w0 + lane;
      if (w < n_win1) {
        const int wy = w / H2, wx = w - wy * H2;
        float p[4][4];
#pragma unroll
        for (int dy = 0; dy < 4; ++dy) {
          const float2* rowp = reinterpret_cast<const float2*>(img + (2 * wy + dy) * kImgW + 2 * wx);
          const float2 u = rowp[0], v = rowp[1];
          p[dy][0] = u.x, p[dy][1] = u.y, p[dy][2] = v.x, p[dy][3] = v.y;
        }
#pragma unroll
        for (int c = 0; c < kC1; ++c) {
          float o00 = 0.f, o01 = 0.f, o10 = 0.f, o11 = 0.f;
#pragma unroll
          for (int dy = 0; dy < 3; ++dy)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx) {
              const float wv = w1r[dy * 3 + dx][c];
              o00 = fmaf(p[dy][dx], wv, o00);
              o01 = fmaf(p[dy][dx + 1], wv, o01);
              o10 = fmaf(p[dy + 1][dx], wv, o10);
              o11 = fmaf(p[dy + 1][dx + 1], wv, o11);
            }
          const float v = fmaxf(fmaxf(fmaxf(o00, o01), fmaxf(o10, o11)) + bias1[c], 0.f);
          a1[c * kA1Plane + (wy + 1) * kA1W + wx + 1] = v;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- conv2 + ReLU + pool on the matrix cores ---------------------------------------------
    for (int g0 = 0; g0 < n_win2; g0 += 4) {
      // A role: row r = lane & 15 -> window g0 + (r >> 2), pixel r & 3; k group = lane >> 4
      const int r = lane & 15;
      const int gA = min(g0 + (r >> 2), n_win2 - 1);
      const int wyA = gA / H4, wxA = gA - wyA * H4;
      const float* base = a1 + q * kA1Plane + (2 * wyA + ((r >> 1) & 1)) * kA1W + 2 * wxA + (r & 1);
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < 18; ++st) {
        const int tap = st >> 1, dy = tap / 3, dx = tap - 3 * dy;
        const float av = base[(4 * (st & 1)) * kA1Plane + dy * kA1W + dx];
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, w2r[st], acc, 0, 0, 0);
      }
      // D role: the four registers of lane (q, n) are window g0 + q of channel n
      const int gD = g0 + q;
      if (gD < n_win2) {
        const float v = fmaxf(fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3])) + bias2, 0.f);
        a2[gD * kC2 + n] = v;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- dense: lane takes features lane, lane + 64, ...; all classes per lane -------------
    float logit[kMaxCls];
#pragma unroll
    for (int c = 0; c < kMaxCls; ++c) logit[c] = 0.f;
    for (int f = lane; f < n_feat; f += 64) {
      const float x = a2[f];
      const float* wrow = Wd + f * n_cls;
#pragma unroll
      for (int c = 0; c < kMaxCls; ++c)
        if (c < n_cls) logit[c] = fmaf(x, wrow[c], logit[c]);
    }
#pragma unroll
    for (int c = 0; c < kMaxCls; ++c)
      if (c < n_cls) logit[c] = wave_sum64(logit[c]) + bd[c];

    if (a.out) {
      float* dst = a.out + (static_cast<size_t>(member) * a.B + im) * n_cls;
#pragma unroll
      for (int c = 0; c < kMaxCls; ++c)
        if (c < n_cls && lane == c) dst[c] = logit[c];
    } else {
      const int y = a.labels[im];  // a label outside [0, n_cls) selects class 0
      float mx = logit[0], picked = logit[0];
#pragma unroll
      for (int c = 1; c < kMaxCls; ++c)
        if (c < n_cls) {
          mx = fmaxf(mx, logit[c]);
          picked = (c == y) ? logit[c] : picked;
        }
      float se = 0.f;
#pragma unroll
      for (int c = 0; c < kMaxCls; ++c)
        if (c < n_cls) se += expf(logit[c] - mx);
      loss_sum += (mx + logf(se)) - picked;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  if (a.partial) {
    if (lane == 0) wave_loss[wave] = loss_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.f;
      for (int w = 0; w < kConvWaves; ++w) t += wave_loss[w];
      a.partial[static_cast<size_t>(member) * a.chunks + blockIdx.x] = t;
    }
  }
}

int convnet_supported(const ConvShape& sh) {
  EVO_REQUIRE(sh.c1 == kC1 && sh.c2 == kC2, EVO_ERR_UNSUPPORTED,
              "convnet: only c1 = %d, c2 = %d are supported (got %d, %d)", kC1, kC2, sh.c1, sh.c2);
  EVO_REQUIRE(sh.H <= kHMax, EVO_ERR_UNSUPPORTED, "convnet: H must be <= %d (got %d)", kHMax, sh.H);
  EVO_REQUIRE(sh.n_cls <= kMaxCls, EVO_ERR_UNSUPPORTED, "convnet: at most %d classes (got %d)", kMaxCls, sh.n_cls);
  return EVO_OK;
}

// Workgroups per member: enough to fill the chip several times over, but no fewer than one
// image per wave.
int convnet_chunks(const ConvShape&, int pop, int B) {
  int chunks = (2048 + pop - 1) / pop;
  const int max_chunks = (B + kConvWaves - 1) / kConvWaves;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  return chunks;
}

int launch_convnet_f32(const ConvShape& sh, const float* params, const float* images, int pop, int B, float* out,
                       const int32_t* labels, float* partial, int chunks, hipStream_t s) {
  ConvArgs a;
  a.params = params, a.images = images, a.labels = labels, a.out = out, a.partial = partial;
  a.P = sh.P, a.H = sh.H, a.n_cls = sh.n_cls, a.B = B;
  if (chunks <= 0) chunks = convnet_chunks(sh, pop, B);
  a.chunks = chunks;
  a.imgs_per_chunk = (B + chunks - 1) / chunks;
  hipLaunchKernelGGL(convnet_kernel, dim3(chunks, pop), dim3(64 * kConvWaves), 0, s, a);
  return check_launch("convnet_kernel");
}

}  // namespace evo
