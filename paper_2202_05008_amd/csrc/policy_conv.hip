// Population-batched fp32 ConvNet forward with a fused cross-entropy epilogue: the image
// classifier of the paper's MNIST example (Section 3, "Supervised Learning Tasks": a
// ConvNet of ~10K parameters trained as a single-step task) evaluated for every member
// with its own weights on one shared batch (Section 2, "Global Policy").
//
// conv3x3 -> ReLU -> maxpool2 -> conv3x3 -> ReLU -> maxpool2 -> dense, c1 = 8, c2 = 16.
//
// Each wavefront runs whole images end to end out of its private 10 KB slice of LDS, with no
// workgroup barrier in the loop: conv1 (K = 9) on the vector ALU, conv2 (K = 72, N = 16:
// 78% of the flops) as implicit GEMM on the matrix cores, the dense layer on the vector ALU
// against a workgroup-shared LDS copy of its weights.  The next image is prefetched into
// registers while the current one is computed.  Activations never leave the chip; per image
// the kernel reads 3 KB (L2 resident, shared by all members).
//
// conv2 arithmetic.  On gfx950 a wave64 fp32 FMA issues every ~2.7 cycles (64 MACs) and
// v_mfma_f32_16x16x4_f32 takes 32 cycles (1024 MACs), and the two do not overlap, so the fp32
// matrix instruction is only 1.4x the vector rate.  v_mfma_f32_16x16x32_f16 takes 16 cycles
// for 8192 MACs.  conv2 therefore runs on the fp16 matrix instruction with every fp32 operand
// split into two half-precision terms (split16.h): three matrix instructions per product, a
// product within 3 * 2^-22 of the fp32 one, a 72-term sum well inside the 1e-5 gate (measured:
// 4e-7 of the rms), at 3 / 16 of the issue cycles of the fp32 matrix instruction.  Both operands
// carry a power-of-two scale chosen at run time so that any finite value fits fp16's range: the
// conv2 weights of a member from their largest magnitude, the conv1 activations of an image from
// the bound max|pixel| max_c sum_t |W1[t][c]| + max_c |b1[c]| (the conv1 sums start from the bias,
// so the factor is one multiply before the ReLU; the conv2 bias is added by the multiply-add that
// takes both factors out again).  A member with a non-finite convolution weight, or an image with
// an infinite pixel, gets NaN logits (the maximum operations of ReLU and pooling would otherwise
// swallow what fp32 arithmetic propagates); a NaN pixel is not detected.
//
// Band pipeline.  conv2 output row b needs the pooled conv1 rows 2b-1 .. 2b+2 only (rows -1 and
// H/2 are the zero border), so the conv1 output is never held whole: pass b of conv1 produces the
// pooled rows 2b and 2b+1 and stores each twice, as rows 1, 2 of the four-row buffer of band b
// and as row 3 of band b-1 and row 0 of band b+1 (three buffers in rotation); conv2 of band b-1
// follows pass b.  H/4 passes do exactly the H/2 rows.  The conv2 output overwrites the part of the
// image buffer that conv1 has already consumed.
//
// conv2 tiling.  The 16 rows of a matrix tile are 4 pooling windows x their 4 pixels, so
// that the 4 accumulator registers of a lane (rows 4q..4q+3 of column n) are exactly one
// pooling window of output channel n: max-pooling is three v_max on registers.  The
// contraction index k = tap * 8 + channel, padded from 72 to 96 = 3 steps of 32 with zero
// weights; lane group q supplies the 8 channels of tap 4 step + q: one 16-byte LDS read per
// split term from the band buffer, which holds [term][row pair][column][row parity][channel]
// half-precision values.
#include "kernels.h"
#include "split16.h"

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr float kFltMax = 3.402823466e+38f;

constexpr int kC1 = 8, kC2 = 16;
constexpr int kHMax = 28;
constexpr int kImgW = kHMax + 2;                     // padded image row (30)
constexpr int kImgFloats = kImgW * kImgW + 4;        // 904: padded image; its consumed part takes the conv2 output
constexpr int kBandW = kHMax / 2 + 2;                // padded conv1-output row (16 pixels)
constexpr int kPixBytes = 2 * kC1;                   // 16: the 8 channels of a pixel as fp16
constexpr int kBandRowPair = 2 * kBandW * kPixBytes;  // 512 bytes: rows 2a and 2a+1, interleaved pixel by pixel
constexpr int kBandTerm = 2 * kBandRowPair;          // 1024 bytes: four rows of one split term
constexpr int kBandBytes = 2 * kBandTerm;            // 2048 bytes per band buffer
constexpr int kBandFloats = kBandBytes / 4;          // 512
constexpr int kWaveFloats = kImgFloats + 3 * kBandFloats;  // 2440 floats = 9,760 bytes per wave

// Byte offset of pixel (row, col) inside one term of a band buffer.  The pixels of an even row and
// of the odd row below it alternate (32 bytes per column), so that the sixteen 16-byte reads of
// a matrix A operand (4 windows x 2 x 2 pixels, any tap) fall on 64 different LDS banks.
__device__ __forceinline__ constexpr int band_off(int row, int col) {
  return (row >> 1) * kBandRowPair + col * 2 * kPixBytes + (row & 1) * kPixBytes;
}
constexpr int kConvWavesMax = 12;
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

// Reductions over the 16 lanes of a row with DPP moves (xor 1, xor 2, half-row mirror, row mirror):
// no LDS round trip, every lane of the row ends with the result, the order is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);  // row_half_mirror
  v += dpp_mov<0x140>(v);  // row_mirror
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  return v;
}

// NCS: row stride of the staged dense weights and number of per-lane class accumulators
// (10 for the ten-class case, 16 for any n_cls <= 16 with zero padding).
// kConvWaves: waves per workgroup (12 with ten classes, 10 when the padded dense weights take 49 KB).
template <int NCS, int kConvWaves>
__global__ __launch_bounds__(64 * kConvWaves) void convnet_kernel(ConvArgs a) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ float wave_loss[kConvWavesMax];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int member = blockIdx.y;
  const int H = a.H, H2 = H / 2, H4 = H / 4;
  const int n_win2 = H4 * H4;  // pooled outputs of conv2
  const int n_feat = n_win2 * kC2;
  const int n_cls = a.n_cls;

  float* wd_s = lds;                                   // [n_feat][NCS] dense weights, shared by the waves
  float* img = lds + kMaxFeat * NCS + wave * kWaveFloats;
  float* band = img + kImgFloats;                      // three band buffers of conv1 output
  float* a2 = img;                                     // conv2 output reuses the consumed image rows

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

  // conv2 weights as matrix B operands, w2b[term][step]: lane group q holds tap 4 step + q (zero
  // beyond tap 8), element j = input channel j, column n; each weight split into two terms
  const int n = lane & 15, q = lane >> 4;
  f16x8 w2b[2][3];
  float u_w2;           // 1 / (scale of the stored conv2 weights)
  bool lane_bad = false;  // a non-finite convolution weight seen by this lane
  {
    float x[3][8];
    float w2_max = 0.f;
#pragma unroll
    for (int st = 0; st < 3; ++st) {
      const int tap = 4 * st + q;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[st][j] = tap < 9 ? W2[(tap * kC1 + j) * kC2 + n] : 0.f;
        w2_max = fmaxf(w2_max, fabsf(x[st][j]));
        lane_bad |= !(fabsf(x[st][j]) <= kFltMax);
      }
    }
    const float s_w2 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(wave_max(w2_max)))));
    u_w2 = pow2_reciprocal(s_w2);
#pragma unroll
    for (int st = 0; st < 3; ++st) {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[st][j] *= s_w2;
      split2_x8(x[st], w2b[0][st], w2b[1][st]);
    }
  }
  const float bias2 = b2[n];
  const float bias_d = (lane & 15) < n_cls ? bd[lane & 15] : 0.f;

  // conv1 role of this lane: pooled pixel (row select rs, column wx) x four channels 4 cg .. 4 cg + 3
  const int c1_win = lane % (2 * H2), c1_cg = min(lane / (2 * H2), 1);
  const bool c1_on = lane < 4 * H2;
  const int c1_rs = c1_win / H2, c1_wx = c1_win - c1_rs * H2;
  float w1v[9][4], bias1v[4];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int c = 0; c < 4; ++c) w1v[t][c] = W1[t * kC1 + 4 * c1_cg + c];
#pragma unroll
  for (int c = 0; c < 4; ++c) bias1v[c] = b1[4 * c1_cg + c];
  // bound on the conv1 activations of any image: max|pixel| * bound_w1 + bound_b1 (both channel groups are
  // present among the lanes of a wave)
  float bound_w1, bound_b1;
  {
    float sw = 0.f, sb = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float t_sum = 0.f;
#pragma unroll
      for (int t = 0; t < 9; ++t) t_sum += fabsf(w1v[t][c]);
      sw = fmaxf(sw, t_sum);
      sb = fmaxf(sb, fabsf(bias1v[c]));
      lane_bad |= !(t_sum <= kFltMax) || !(fabsf(bias1v[c]) <= kFltMax) || !(fabsf(bias2) <= kFltMax);
    }
    bound_w1 = wave_max(sw);
    bound_b1 = wave_max(sb);
  }
  const bool member_bad = __any(lane_bad);

  // conv2 A role of this lane: row r = lane & 15 -> window 4 h + (r >> 2) of the band, pixel r & 3,
  // shifted by tap 4 step + q (the padding taps 9..11 re-read tap 8 against zero weights)
  int a_off[2][3];  // bytes from the start of a band buffer
  {
    const int r = lane & 15, i = r & 3;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int wxA = min(4 * h + (r >> 2), H4 - 1);
#pragma unroll
      for (int st = 0; st < 3; ++st) {
        const int tap = min(4 * st + q, 8), dy = tap / 3, dx = tap - 3 * dy;
        a_off[h][st] = band_off((i >> 1) + dy, 2 * wxA + (i & 1) + dx);
      }
    }
  }
  char* const bandb = reinterpret_cast<char*>(band);
  // conv1 store targets of this lane inside a band buffer: its row of the pass (2b or 2b+1) is row
  // 1 or 2 of band b and row 3 of band b-1 or row 0 of band b+1
  const int c1_dst_own = band_off(1 + c1_rs, c1_wx + 1) + 8 * c1_cg;
  const int c1_dst_nbr = band_off(c1_rs ? 0 : 3, c1_wx + 1) + 8 * c1_cg;
  // one padded band row (16 pixels of 16 bytes, both terms) set to zero by lanes 0..31
  auto zero_band_row = [&](char* buf, int row) {
    if (lane < 32) *reinterpret_cast<uint4*>(buf + (lane >> 4) * kBandTerm + band_off(row, lane & 15)) = make_uint4(0, 0, 0, 0);
  };

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
    float px_max = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = lane + 64 * j;
      if (i < n_vec) {
        const int y = i / row4, x4 = i - y * row4;
        float* d = img + (y + 1) * kImgW + 4 * x4 + 1;
        d[0] = pre[j].x, d[1] = pre[j].y, d[2] = pre[j].z, d[3] = pre[j].w;
        px_max = fmaxf(fmaxf(fmaxf(px_max, fabsf(pre[j].x)), fabsf(pre[j].y)), fmaxf(fabsf(pre[j].z), fabsf(pre[j].w)));
      }
    }
    // scale of this image's conv1 activations from the bound on them, and the factor that takes it and the
    // weights' scale out again (all wave-uniform; non-negative floats order like their bit patterns)
    px_max = row16_max(px_max);
    const uint32_t px_bits = max(max(__builtin_amdgcn_readlane(__float_as_uint(px_max), 0),
                                     __builtin_amdgcn_readlane(__float_as_uint(px_max), 16)),
                                 max(__builtin_amdgcn_readlane(__float_as_uint(px_max), 32),
                                     __builtin_amdgcn_readlane(__float_as_uint(px_max), 48)));
    const float a1_bound = fmaf(__uint_as_float(px_bits), bound_w1, bound_b1);
    const float s_a1 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(a1_bound))));
    const float u_a2 = pow2_reciprocal(s_a1) * u_w2;
    const bool image_bad = member_bad || !(a1_bound <= kFltMax);
    if (im + kConvWaves < img_end) {
      const float4* src = reinterpret_cast<const float4*>(a.images + static_cast<size_t>(im + kConvWaves) * H * H);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (lane + 64 * j < n_vec) pre[j] = src[lane + 64 * j];
    }
    wave_sync();

    zero_band_row(bandb, 0);  // band 0, row 0: the border above the image
    int b3 = 0;               // b mod 3: buffer of band b
#pragma unroll 1
    for (int b = 0; b <= H4; ++b) {
      // ---- conv1 + ReLU + pool, pass b: pooled rows 2b and 2b+1 ----
      if (b == H4) {
        zero_band_row(bandb + (b3 == 0 ? 2 : b3 - 1) * kBandBytes, 3);  // last band, row 3: the border below the image
      } else if (c1_on) {
        const int pr = 2 * b + c1_rs;  // pooled row of this lane
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        {
          float p[4][4];
#pragma unroll
          for (int dy = 0; dy < 4; ++dy) {
            const float2* rowp = reinterpret_cast<const float2*>(img + (2 * pr + dy) * kImgW + 2 * c1_wx);
            const float2 u = rowp[0], w = rowp[1];
            p[dy][0] = u.x, p[dy][1] = u.y, p[dy][2] = w.x, p[dy][3] = w.y;
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            float o00 = bias1v[c], o01 = o00, o10 = o00, o11 = o00;
#pragma unroll
            for (int dy = 0; dy < 3; ++dy)
#pragma unroll
              for (int dx = 0; dx < 3; ++dx) {
                const float wv = w1v[dy * 3 + dx][c];
                o00 = fmaf(p[dy][dx], wv, o00);
                o01 = fmaf(p[dy][dx + 1], wv, o01);
                o10 = fmaf(p[dy + 1][dx], wv, o10);
                o11 = fmaf(p[dy + 1][dx + 1], wv, o11);
              }
            v[c] = fmaxf(fmaxf(fmaxf(o00, o01), fmaxf(o10, o11)) * s_a1, 0.f);  // stored times s_a1
          }
        }
        // two fp16 terms of the four channels: 8 bytes per term
        uint2 term[2];
        split2_pair(v[0], v[1], term[0].x, term[1].x);
        split2_pair(v[2], v[3], term[0].y, term[1].y);
        // own band, and the neighbour band that shares the row
        const int nbr3 = c1_rs ? (b3 == 2 ? 0 : b3 + 1) : (b3 == 0 ? 2 : b3 - 1);
        char* cur = bandb + b3 * kBandBytes + c1_dst_own;
        char* nxt = bandb + nbr3 * kBandBytes + c1_dst_nbr;
#pragma unroll
        for (int k = 0; k < 2; ++k) *reinterpret_cast<uint2*>(cur + k * kBandTerm) = term[k];
        if (c1_rs ? b + 1 < H4 : b >= 1) {
#pragma unroll
          for (int k = 0; k < 2; ++k) *reinterpret_cast<uint2*>(nxt + k * kBandTerm) = term[k];
        }
      }
      wave_sync();
      const int prev3 = b3 == 0 ? 2 : b3 - 1;  // buffer of band b - 1
      b3 = b3 == 2 ? 0 : b3 + 1;
      if (b == 0) continue;

      // ---- conv2 + ReLU + pool, band b-1: two independent tiles (windows 0..3 and 4..7 of the row) --
      const char* bb = bandb + prev3 * kBandBytes;
      floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};  // h h'
      floatx4 low0 = {0.f, 0.f, 0.f, 0.f}, low1 = {0.f, 0.f, 0.f, 0.f};  // 2^11 (h m' + m h')
#pragma unroll
      for (int st = 0; st < 3; ++st) {
        f16x8 a0[2], a1[2];  // [term] of tile 0 and tile 1
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          a0[k] = *reinterpret_cast<const f16x8*>(bb + a_off[0][st] + k * kBandTerm);
          a1[k] = *reinterpret_cast<const f16x8*>(bb + a_off[1][st] + k * kBandTerm);
        }
        low0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0[1], w2b[0][st], low0, 0, 0, 0);
        low1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[1], w2b[0][st], low1, 0, 0, 0);
        low0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0[0], w2b[1][st], low0, 0, 0, 0);
        low1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[0], w2b[1][st], low1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0[0], w2b[0][st], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[0], w2b[0][st], acc1, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0[i] = fmaf(low0[i], kSplitLowUnscale, acc0[i]);
        acc1[i] = fmaf(low1[i], kSplitLowUnscale, acc1[i]);
      }
      // D role: the four registers of lane (q, n) are window q (+4) of channel n
      if (q < H4)
        a2[((b - 1) * H4 + q) * kC2 + n] =
            fmaxf(fmaf(fmaxf(fmaxf(acc0[0], acc0[1]), fmaxf(acc0[2], acc0[3])), u_a2, bias2), 0.f);
      if (q + 4 < H4)
        a2[((b - 1) * H4 + q + 4) * kC2 + n] =
            fmaxf(fmaf(fmaxf(fmaxf(acc1[0], acc1[1]), fmaxf(acc1[2], acc1[3])), u_a2, bias2), 0.f);
      wave_sync();
    }

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
    // transpose-reduce through LDS (the band buffers are free now): lane (c, part) adds 16 partials
    float* red = band;
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
    if (image_bad) logit = __builtin_nanf("");  // a non-finite weight or pixel: what fp32 arithmetic would propagate
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
      const float mx = row16_max(lv);
      const float se = row16_sum(cls < n_cls ? expf(lv - mx) : 0.f);
      const float picked = row16_sum(cls == y ? lv : 0.f);
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

// Workgroups per member: two per compute unit over the whole grid (one resident, one queued, so
// that the per-workgroup staging of the weights is paid rarely), but no fewer than one image per wave.
int convnet_chunks(const ConvShape&, int pop, int B) {
  int chunks = (512 + pop - 1) / pop;
  const int max_chunks = (B + kConvWavesMax - 1) / kConvWavesMax;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  return chunks;
}

template <int NCS, int WAVES>
static int launch_conv(const ConvArgs& a, int pop, hipStream_t s) {
  const size_t shmem = sizeof(float) * (static_cast<size_t>(kMaxFeat) * NCS + WAVES * kWaveFloats);
  static_assert(sizeof(float) * (kMaxFeat * NCS + WAVES * kWaveFloats) + 256 <= 160 * 1024, "LDS budget of a CU");
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(convnet_kernel<NCS, WAVES>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
  if (e != hipSuccess) (void)hipGetLastError();  // do not leave the error sticky for the caller's next HIP call
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((convnet_kernel<NCS, WAVES>), dim3(a.chunks, pop), dim3(64 * WAVES), shmem, s, a);
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
  return sh.n_cls == 10 ? launch_conv<10, 12>(a, pop, s) : launch_conv<16, 10>(a, pop, s);
}

}  // namespace evo
