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
// vector ALU against a workgroup-shared LDS copy of its weights.  The eight waves of a
// workgroup are at different stages, so matrix and vector work overlap on a SIMD.  The next
// image is prefetched into registers while the current one is computed.  Activations never
// leave the chip; per image the kernel reads 3 KB (L2 resident, shared by all members).
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
constexpr int kImgW = kHMax + 2;                     // padded image row (30)
constexpr int kImgFloats = kImgW * kImgW + 4;        // 904: padded image; later the conv2 output (784)
constexpr int kA1W = kHMax / 2 + 2;                  // padded conv1-output row (16)
constexpr int kA1Plane = kA1W * kA1W + 8;            // 264: plane stride = 8 mod 32 banks
constexpr int kA1Floats = kC1 * kA1Plane;            // 2112: conv1 output; later the dense partial sums
constexpr int kWaveFloats = kImgFloats + kA1Floats;  // 3016 floats = 12,064 bytes per wave
constexpr int kConvWaves = 8;
constexpr int kMaxCls = 16;
constexpr int kMaxFeat = (kHMax / 4) * (kHMax / 4) * kC2;  // 784

struct ConvArgs {
  const float* params;
  const float* images;
  const int32_t* labels;
  float* out;
  float* partial;
  int P, H, n_cls, B, chunks, imgs_per_chunk;
};

__device__ __forceinline__ void wave_sync() {
  // LDS traffic of one wave is issued in order; this only stops the compiler from moving
  // accesses of different lanes' data across the point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// NCS: row stride of the staged dense weights and number of per-lane class accumulators
// (10 for the ten-class case, 16 for any n_cls <= 16 with zero padding).
template <int NCS>
__global__ __launch_bounds__(64 * kConvWaves) void convnet_kernel(ConvArgs a) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ float wave_loss[kConvWaves];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int member = blockIdx.y;
  const int H = a.H, H2 = H / 2, H4 = H / 4;
  const int n_win1 = H2 * H2;  // pooled outputs of conv1
  const int n_win2 = H4 * H4;  // pooled outputs of conv2
  const int n_feat = n_win2 * kC2;
  const int n_cls = a.n_cls;

  float* wd_s = lds;                                   // [n_feat][NCS] dense weights, shared by the waves
  float* img = lds + kMaxFeat * NCS + wave * kWaveFloats;
  float* a1 = img + kImgFloats;
  float* a2 = img;                                     // conv2 output reuses the image buffer

  const float* theta = a.params + static_cast<size_t>(member) * a.P;
  const float* W1 = theta;                 // [3][3][1][8]
  const float* b1 = theta + 9 * kC1;       // [8]
  const float* W2 = b1 + kC1;              // [3][3][8][16]
  const float* b2 = W2 + 9 * kC1 * kC2;    // [16]
  const float* Wd = b2 + kC2;              // [n_feat][n_cls]
  const float* bd = Wd + n_feat * n_cls;   // [n_cls]

  // ---- once per workgroup: dense weights -> LDS (rows padded to NCS with zeros) ----------------
  for (int i = threadIdx.x; i < n_feat * NCS; i += 64 * kConvWaves) {
    const int f = i / NCS, c = i - f * NCS;
    wd_s[i] = c < n_cls ? Wd[f * n_cls + c] : 0.f;
  }
  // zero the padded buffers once: borders stay zero, interiors are overwritten per image
  for (int i = lane; i < kWaveFloats; i += 64) img[i] = 0.f;

  // conv2 weights as matrix B operands: 18 steps, k = 4 step + q, column n
  const int n = lane & 15, q = lane >> 4;
  float w2r[18];
#pragma unroll
  for (int st = 0; st < 18; ++st) w2r[st] = W2[(4 * st + q) * kC2 + n];
  const float bias2 = b2[n];
  const float bias_d = (lane & 15) < n_cls ? bd[lane & 15] : 0.f;

  const int img_begin = blockIdx.x * a.imgs_per_chunk;
  const int img_end = min(a.B, img_begin + a.imgs_per_chunk);
  const int row4 = H / 4, n_vec = H * row4;  // float4 pieces of one image (<= 196)
  float loss_sum = 0.f;

  // prefetch of the first image: lane takes pieces lane, lane + 64, ...
  float4 pre[4];
  int im = img_begin + wave;
  if (im < img_end) {
    const float4* src = reinterpret_cast<const float4*>(a.images + static_cast<size_t>(im) * H * H);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j < n_vec) pre[j] = src[lane + 64 * j];
  }
  __syncthreads();  // dense weights staged

  for (; im < img_end; im += kConvWaves) {
    // ---- image registers -> zero-padded LDS buffer; then prefetch the next image ---------------
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = lane + 64 * j;
      if (i < n_vec) {
        const int y = i / row4, x4 = i - y * row4;
        float* d = img + (y + 1) * kImgW + 4 * x4 + 1;
        d[0] = pre[j].x, d[1] = pre[j].y, d[2] = pre[j].z, d[3] = pre[j].w;
      }
    }
    if (im + kConvWaves < img_end) {
      const float4* src = reinterpret_cast<const float4*>(a.images + static_cast<size_t>(im + kConvWaves) * H * H);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (lane + 64 * j < n_vec) pre[j] = src[lane + 64 * j];
    }
    wave_sync();

    // ---- conv1 + ReLU + pool: lane = pooled output pixel; two passes of four channels so that
    //      the 40 wave-uniform weights of a pass fit in scalar registers --------------------------
#pragma unroll 1
    for (int cg = 0; cg < 2; ++cg) {
      float w1r[9][4], bias1[4];
#pragma unroll
      for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int c = 0; c < 4; ++c) w1r[t][c] = W1[t * kC1 + 4 * cg + c];
#pragma unroll
      for (int c = 0; c < 4; ++c) bias1[c] = b1[4 * cg + c];
#pragma unroll 1
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
          for (int c = 0; c < 4; ++c) {
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
            a1[(4 * cg + c) * kA1Plane + (wy + 1) * kA1W + wx + 1] = v;
          }
        }
      }
    }
    wave_sync();
    // ---- conv2 + ReLU + pool on the matrix cores, two independent tiles per pass ---------------
    for (int g0 = 0; g0 < n_win2; g0 += 8) {
      // A role: row r = lane & 15 -> window g0 + (r >> 2), pixel r & 3; k group = lane >> 4
      const int r = lane & 15;
      const float* base[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int gA = min(g0 + 4 * h + (r >> 2), n_win2 - 1);
        const int wyA = gA / H4, wxA = gA - wyA * H4;
        base[h] = a1 + q * kA1Plane + (2 * wyA + ((r >> 1) & 1)) * kA1W + 2 * wxA + (r & 1);
      }
      floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < 18; ++st) {
        const int tap = st >> 1, dy = tap / 3, dx = tap - 3 * dy;
        const int o = (4 * (st & 1)) * kA1Plane + dy * kA1W + dx;
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(base[0][o], w2r[st], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(base[1][o], w2r[st], acc1, 0, 0, 0);
      }
      // D role: the four registers of lane (q, n) are window g0 + q (+4) of channel n.  The
      // writes go to the image buffer, whose last reader (conv1) is done.
      const int gD0 = g0 + q, gD1 = g0 + 4 + q;
      if (gD0 < n_win2)
        a2[gD0 * kC2 + n] = fmaxf(fmaxf(fmaxf(acc0[0], acc0[1]), fmaxf(acc0[2], acc0[3])) + bias2, 0.f);
      if (gD1 < n_win2)
        a2[gD1 * kC2 + n] = fmaxf(fmaxf(fmaxf(acc1[0], acc1[1]), fmaxf(acc1[2], acc1[3])) + bias2, 0.f);
    }
    wave_sync();

    // ---- dense: lane takes features lane, lane + 64, ... and accumulates every class ---------
    float acc[NCS];
#pragma unroll
    for (int c = 0; c < NCS; ++c) acc[c] = 0.f;
    for (int f = lane; f < n_feat; f += 64) {
      const float x = a2[f];
      const float* wrow = wd_s + f * NCS;
#pragma unroll
      for (int c = 0; c < NCS; ++c) acc[c] = fmaf(x, wrow[c], acc[c]);
    }
    // transpose-reduce through LDS (conv1's buffer is free now): lane (c, part) adds 16 partials
    float* red = a1;
#pragma unroll
    for (int c = 0; c < NCS; ++c) red[lane * NCS + c] = acc[c];
    wave_sync();
    float logit = 0.f;
    {
      const int c = lane & 15, part = lane >> 4;
      if (c < NCS) {
#pragma unroll
        for (int i = 0; i < 16; ++i) logit += red[(16 * part + i) * NCS + c];
      }
      logit += __shfl_xor(logit, 16, 64);
      logit += __shfl_xor(logit, 32, 64);
      logit += bias_d;
    }
    wave_sync();
    // both scratch uses sat on zero-padded buffers: restore the zeros (the next image's
    // interior is rewritten anyway, the borders must read as zero again)
    for (int i = lane; i < 64 * NCS; i += 64) red[i] = 0.f;
    for (int i = lane; i < n_feat; i += 64) a2[i] = 0.f;

    const int cls = lane & 15;
    if (a.out) {
      if (lane < n_cls) a.out[(static_cast<size_t>(member) * a.B + im) * n_cls + lane] = logit;
    } else {
      // cross-entropy over the 16 lanes of a row (classes beyond n_cls count as -inf)
      const int y = a.labels[im];  // a label outside [0, n_cls) contributes logit 0
      const float lv = cls < n_cls ? logit : -INFINITY;
      float mx = lv;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      float se = cls < n_cls ? expf(lv - mx) : 0.f;
      float picked = cls == y ? lv : 0.f;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) {
        se += __shfl_xor(se, off, 64);
        picked += __shfl_xor(picked, off, 64);
      }
      loss_sum += (mx + logf(se)) - picked;
    }
    wave_sync();
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

template <int NCS>
static int launch_conv(const ConvArgs& a, int pop, hipStream_t s) {
  const size_t shmem = sizeof(float) * (static_cast<size_t>(kMaxFeat) * NCS + kConvWaves * kWaveFloats);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(convnet_kernel<NCS>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
  hipLaunchKernelGGL(convnet_kernel<NCS>, dim3(a.chunks, pop), dim3(64 * kConvWaves), shmem, s, a);
  return check_launch("convnet_kernel");
}

int launch_convnet_f32(const ConvShape& sh, const float* params, const float* images, int pop, int B, float* out,
                       const int32_t* labels, float* partial, int chunks, hipStream_t s) {
  ConvArgs a;
  a.params = params, a.images = images, a.labels = labels, a.out = out, a.partial = partial;
  a.P = sh.P, a.H = sh.H, a.n_cls = sh.n_cls, a.B = B;
  if (chunks <= 0) chunks = convnet_chunks(sh, pop, B);
  a.chunks = chunks;
  a.imgs_per_chunk = (B + chunks - 1) / chunks;
  return sh.n_cls == 10 ? launch_conv<10>(a, pop, s) : launch_conv<16>(a, pop, s);
}

}  // namespace evo
