// Population-batched fp32 ConvNet forward with a fused cross-entropy epilogue: the image
// classifier of the paper's MNIST example (Section 3, "Supervised Learning Tasks": a
// ConvNet of ~10K parameters trained as a single-step task) evaluated for every member
// with its own weights on one shared batch (Section 2, "Global Policy").
//
// conv3x3 -> ReLU -> maxpool2 -> conv3x3 -> ReLU -> maxpool2 -> dense, c1 = 8, c2 = 16.
//
// Each wavefront runs whole images end to end out of its private 8.75 KB slice of LDS, with no
// workgroup barrier in the loop: both convolutions as implicit GEMMs on the matrix cores, the dense layer
// on the vector ALU against a workgroup-shared LDS copy of its weights, accumulated band by band from the
// conv2 results while they are still in registers.  The next image is prefetched into
// registers while the current one is computed.  Activations never leave the chip.  The conversion of the images into
// the two fp16 planes conv1 reads is the same for every member: for roll-outs a small kernel does it once per batch
// into the caller's workspace (4 KB per image, L2 resident, read by all members; 8 % of the ConvNet kernel's time
// when every member's workgroups did it again), pop_forward, which has no workspace, converts in the kernel.
//
// Arithmetic.  On gfx950 a wave64 fp32 FMA issues every ~2.7 cycles (64 MACs) and
// v_mfma_f32_16x16x4_f32 takes 32 cycles (1024 MACs), and the two do not overlap, so the fp32
// matrix instruction is only 1.4x the vector rate.  v_mfma_f32_16x16x32_f16 takes 16 cycles
// for 8192 MACs.  The convolutions therefore run on the fp16 matrix instruction with every fp32 operand
// split into two half-precision terms (split16.h): a product within 3 * 2^-22 of the fp32 one, sums of 9 and
// 72 terms well inside the 1e-5 gate (measured: 2e-7 .. 7e-7 of the rms of the logits).  Every operand
// carries a power-of-two scale chosen at run time so that any finite value fits fp16's range: the
// weights of a member from their largest magnitude (conv1: per output channel), the pixels of an image from
// their largest magnitude, the conv1 activations of an image from
// the bound max|pixel| max_c sum_t |W1[t][c]| + max_c |b1[c]| (the sums of both convolutions start from the bias in
// their own units, so the factor back is one multiply after ReLU and pooling; the scales are limited where a bias is
// more than 2^70 times the convolution it is added to, so that this start value stays finite).  A member with a non-finite convolution weight, or an image with
// an infinite pixel, gets NaN logits (the maximum operations of ReLU and pooling would otherwise
// swallow what fp32 arithmetic propagates); a NaN pixel is not detected.
//
// conv1 tiling (K = 9, one input channel).  The image sits in LDS as two planes of fp16 terms, the padded rows 2 k
// and 2 k + 1 interleaved pixel by pixel (written with aligned 16-byte stores: a lane gets the column left of its
// four from the lane before it), so that the eight values a lane contributes to a patch are 16 consecutive bytes.  The 16
// columns of a matrix tile are 16 pooling windows (8 window columns x the two pooled rows of the pass); the contraction runs over the 4 x 4 pixel patch that holds
// the 3 x 3 neighbourhoods of the window's four pixels (the lane's eight values are four consecutive columns of a
// row pair: one LDS instruction of two 8-byte reads), once against the leading terms of the pixels (lane groups
// 0, 1) and once against their residual terms (lane groups 2, 3), which fills K = 32.  The 16 rows are
// (8 output channels) x (the window's two pixel columns); one set of weight operands per pixel row of the
// window (the stencil shifted inside the patch, zeros elsewhere).  With the residual terms stored as they are
// (split16.h: the matrix instruction keeps half-precision subnormals), h h' + m' h + h' m takes two
// instructions into ONE accumulator: (h | h) and (m | 0) against (h' | m').  Row order (channel pair, column, channel parity) puts a window's two columns of channels
// 2 q, 2 q + 1 into the four accumulator registers of lane group q: pooling is three maxima per channel on
// registers; one swap between neighbouring lane groups and one between the halves of the wave then collect a
// window's four channel pairs, and the pooled pixel goes to the band buffers as one 16-byte store per term.
// (LDS counters decided these two layouts: 2-byte stores of the image and 4-byte stores of the channel pairs,
// at 32 bytes from window to window, cost 14 % and 15 % of the kernel's time in bank and address conflicts.)
//
// Band pipeline.  conv2 output row b needs the pooled conv1 rows 2b-1 .. 2b+2 only (rows -1 and
// H/2 are the zero border), so the conv1 output is never held whole: pass b of conv1 produces the
// pooled rows 2b and 2b+1 and stores them into a ring of eight rows (plus copies of two of them, so that the four
// rows of a band always lie at consecutive addresses); conv2 of band b-1 follows pass b.  The loop is written out
// four passes at a time, which makes every ring address a lane constant plus an immediate of the LDS
// instruction.  H/4 passes do exactly the H/2 rows.  The conv2 output never goes to memory: its pooled
// values are the dense layer's features and are consumed from the registers they are computed in.
//
// conv2 tiling.  One matrix tile covers a whole band: its 16 rows are the 16 pixel columns of the (padded)
// conv2 output row pair, i.e. 8 pooling windows x their two columns, and the two pixel rows of the windows
// are two accumulators that share the A operands.  The contraction of one step is (4 band rows) x (8 input
// channels) for one tap column kx: lane group q supplies band row q, and the weights of output row py sit in lane
// group q as tap row ky = q - py (zero where that falls outside the stencil: a quarter of each operand), so the
// second output row costs a second set of weight registers and no LDS traffic.  Lane (q, r) therefore reads the
// pixel (band row q, column r + kx): ONE 16-byte read per split term gives tap column 0, conflict-free (the 64
// lanes read 1 KB end to end), and tap columns 1 and 2 are the values of the lanes one and two further
// (row_shl moves).  Two reads per band instead of the twelve of an im2col read per tap (measured: LDS busy
// 78 % -> 66 %).  The 4 accumulator registers of lane (q, n) are the two columns of windows 2 q and 2 q + 1 of
// output channel n: with the second accumulator, max-pooling is in-lane.  The sums start from the bias in their
// own units, so ReLU and pooling are integer maxima on the bit patterns, as for conv1.
#include "kernels.h"
#include "split16.h"
#include <type_traits>

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr float kFltMax = 3.402823466e+38f;

constexpr int kC1 = 8, kC2 = 16;
constexpr int kHMax = 28;
// A split term of the padded image: padded rows 2 k and 2 k + 1 interleaved pixel by pixel (4 bytes per column),
// so that the two rows x four columns of a conv1 patch operand are 16 consecutive bytes.
constexpr int kPairPitch = 128;                      // bytes of a row pair: 30 columns x 2 rows x 2 bytes, 8 spare
constexpr int kPlaneBytes = (kHMax / 2 + 1) * kPairPitch;  // 1920
constexpr int kImgBytes = 2 * kPlaneBytes;           // the padded image as two fp16 terms (3840)
constexpr int kBandW = kHMax / 2 + 2;                // padded conv1-output row (16 pixels)
constexpr int kPixBytes = 2 * kC1;                   // 16: the 8 channels of a pixel as fp16
constexpr int kBandRowPair = 2 * kBandW * kPixBytes;  // 512 bytes: rows 2a and 2a+1, interleaved pixel by pixel
// The pooled conv1 rows live in a ring of eight rows per split term (row (r + 1) mod 8 for pooled row r, so the
// border above the image is row 0), followed by copies of rows 0 and 1 as rows 8 and 9: the four rows of a conv2
// band then always lie at consecutive addresses, starting two rows further with every band and back at row 0
// every fourth one.
constexpr int kRingRows = 10;
constexpr int kBandTerm = (kRingRows / 2) * kBandRowPair;   // 2560 bytes: the ring of one split term
constexpr int kBandBytes = 2 * kBandTerm;            // 5120 bytes
constexpr int kBandFloats = kBandBytes / 4;          // 1280
constexpr int kWaveFloats = kImgBytes / 4 + kBandFloats;  // 2240 floats = 8,960 bytes per wave

// Byte offset of pixel (row, col) inside one term of a band buffer.  The pixels of an even row and
// of the odd row below it alternate (32 bytes per column), so that the sixteen 16-byte reads of
// a matrix A operand (4 windows x 2 x 2 pixels, any tap) fall on 64 different LDS banks.
__device__ __forceinline__ constexpr int band_off(int row, int col) {
  return (row >> 1) * kBandRowPair + col * 2 * kPixBytes + (row & 1) * kPixBytes;
}
constexpr int kConvWavesMax = 12;
// The batch split once for all members (convnet_split_kernel): per image the two padded planes exactly as they sit
// in LDS, then the largest pixel magnitude as a float.
constexpr int kImgStride = 4096;
constexpr int kSplitWaves = 4;
constexpr int kMaxCls = 16;
constexpr int kMaxFeat = (kHMax / 4) * (kHMax / 4) * kC2;  // 784

struct ConvArgs {
  const float* params;
  const float* images;
  const int32_t* labels;
  const unsigned char* planes;  // the batch already split into fp16 terms (kImgStride bytes per image), or null
  float* out;
  float* partial;
  float* fitness;  // with one workgroup per member: fitness[member] = scale * (the member's loss sum), no partial sums
  float scale;
  int P, H, n_cls, B, chunks, imgs_per_chunk;
};

__device__ __forceinline__ void wave_sync() {
  // LDS traffic of one wave is issued in order; this only stops the compiler from moving
  // accesses of different lanes' data across the point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A value moved between the lanes of a row (DPP control CTRL): no LDS round trip.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  // every lane has a source in these patterns: no value has to be prepared for lanes without one
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// Reductions over one quad of every row (lanes 1 and 2 apart) and then down the four rows: lane 63 ends with the
// result over the last quads of the rows (row_bcast:15 hands a row's last lane to the next row, row_bcast:31 the
// second row's to the third and fourth).
__device__ __forceinline__ float quads_sum(float v) {
  v += dpp_mov<0xB1>(v);  // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);  // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xa, 0xf, false));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xc, 0xf, false));
  return v;
}
__device__ __forceinline__ float quads_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x142, 0xa, 0xf, false)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x143, 0xc, 0xf, false)));
  return v;
}
__device__ __forceinline__ float last_lane(float v) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Largest magnitude over the 16 lanes of a row, in every lane of it (non-negative floats order like their bit
// patterns): integer maxima, which take the moved value as an operand and need no canonicalising moves.
__device__ __forceinline__ float row16_max_magnitude(float v) {
  int b = __float_as_int(v);
  b = max(b, __float_as_int(dpp_mov<0xB1>(__int_as_float(b))));
  b = max(b, __float_as_int(dpp_mov<0x4E>(__int_as_float(b))));
  b = max(b, __float_as_int(dpp_mov<0x141>(__int_as_float(b))));
  b = max(b, __float_as_int(dpp_mov<0x140>(__int_as_float(b))));
  return __int_as_float(b);
}

// NCS: row stride of the staged dense weights and number of per-lane class accumulators
// (10 for the ten-class case, 16 for any n_cls <= 16 with zero padding).
// kConvWaves: waves per workgroup (12 with ten classes, 10 when the padded dense weights take 49 KB).
// The pixels of one image (lane's float4 pieces lane, lane + 64, ... of its rows) -> two fp16 terms in the
// zero-padded planes; returns the largest pixel magnitude (wave-uniform).  The pixels' power of two depends on the image alone.
__device__ __forceinline__ float pixel_scale(float px_bound) {
  return __int_as_float(__builtin_amdgcn_readfirstlane(min(__float_as_int(split_pow2_scale(px_bound)) >> 23, 183) << 23));
}
// The lane's pieces of an image: task t = lane + 64 round (round 0, 1) is the row pair k = t / row4 (padded rows
// 2 k and 2 k + 1, i.e. image rows 2 k - 1 and 2 k) and the float4 piece x4 = t % row4 of both rows; pre[2 round]
// and pre[2 round + 1] hold them (zeros for the border rows and for tasks beyond the image).
__device__ __forceinline__ void load_pixels(const float* __restrict__ image, int H, int lane, int row4, float4 (&pre)[4]) {
  const int n_task = (H / 2 + 1) * row4;  // at most 105
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const int t = lane + 64 * round, k = t / row4, x4 = t - k * row4;
    const float4* row_b = reinterpret_cast<const float4*>(image + static_cast<size_t>(2 * k) * H) + x4;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    pre[2 * round] = (t < n_task && k > 0) ? *(row_b - row4) : zero;
    pre[2 * round + 1] = (t < n_task && 2 * k < H) ? *row_b : zero;
  }
}
__device__ __forceinline__ float stage_pixels(const float4 (&pre)[4], char* planes, int lane, int row4, int n_task) {
  float px_max = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    px_max = fmaxf(fmaxf(fmaxf(px_max, fabsf(pre[j].x)), fabsf(pre[j].y)), fmaxf(fabsf(pre[j].z), fabsf(pre[j].w)));
  // (non-negative floats order like their bit patterns)
  px_max = row16_max_magnitude(px_max);
  const uint32_t px_bits = max(max(__builtin_amdgcn_readlane(__float_as_uint(px_max), 0),
                                   __builtin_amdgcn_readlane(__float_as_uint(px_max), 16)),
                               max(__builtin_amdgcn_readlane(__float_as_uint(px_max), 32),
                                   __builtin_amdgcn_readlane(__float_as_uint(px_max), 48)));
  const float px_bound = __uint_as_float(px_bits);
  const float s_px = pixel_scale(px_bound);
  // Pixels 4 x4 .. 4 x4 + 3 of a row sit at padded columns 4 x4 + 1 ..: a task stores the aligned 16 bytes of
  // columns 4 x4 .. 4 x4 + 3 of its row pair (a column = the two rows' pixels), whose first column is the last one
  // of the piece to its left (the lane before it; for lane 0 the last lane of the previous round), and the last
  // piece of a row pair adds the pair's last column.
  uint32_t last_lead = 0, last_resid = 0;  // lane 63's last column of the previous round
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const int t = lane + 64 * round, k = t / row4, x4 = t - k * row4;
    const float4 ra = pre[2 * round], rb = pre[2 * round + 1];
    uint32_t lead[4], resid[4];  // columns x, y, z, w of the piece: (upper row, lower row) as a pair of fp16
    split2_pair_true(ra.x * s_px, rb.x * s_px, lead[0], resid[0]);
    split2_pair_true(ra.y * s_px, rb.y * s_px, lead[1], resid[1]);
    split2_pair_true(ra.z * s_px, rb.z * s_px, lead[2], resid[2]);
    split2_pair_true(ra.w * s_px, rb.w * s_px, lead[3], resid[3]);
    uint32_t left_lead = __builtin_amdgcn_update_dpp(last_lead, lead[3], 0x138, 0xf, 0xf, false);    // wave_shr:1
    uint32_t left_resid = __builtin_amdgcn_update_dpp(last_resid, resid[3], 0x138, 0xf, 0xf, false);
    last_lead = __builtin_amdgcn_readlane(lead[3], 63);
    last_resid = __builtin_amdgcn_readlane(resid[3], 63);
    if (x4 == 0) left_lead = 0, left_resid = 0;  // the border left of the rows
    if (t < n_task) {
      char* d = planes + k * kPairPitch + 16 * x4;
      *reinterpret_cast<uint4*>(d) = make_uint4(left_lead, lead[0], lead[1], lead[2]);
      *reinterpret_cast<uint4*>(d + kPlaneBytes) = make_uint4(left_resid, resid[0], resid[1], resid[2]);
      if (x4 == row4 - 1) {
        *reinterpret_cast<uint32_t*>(d + 16) = lead[3];
        *reinterpret_cast<uint32_t*>(d + kPlaneBytes + 16) = resid[3];
      }
    }
  }
  return px_bound;
}

// Once per batch, for all members: every image as its two padded fp16 planes plus its largest pixel magnitude.
// One wave per image at a time, through the same LDS staging as the ConvNet kernel's own.
__global__ __launch_bounds__(64 * kSplitWaves) void convnet_split_kernel(const float* __restrict__ images, int B, int H,
                                                                         unsigned char* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) char planes_s[kSplitWaves][kImgBytes];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* planes = planes_s[wave];
  for (int i = lane; i < kImgBytes / 16; i += 64) reinterpret_cast<uint4*>(planes)[i] = make_uint4(0, 0, 0, 0);
  wave_sync();
  const int row4 = H / 4, n_task = (H / 2 + 1) * row4;
  for (int im = blockIdx.x * kSplitWaves + wave; im < B; im += gridDim.x * kSplitWaves) {
    float4 pre[4];
    load_pixels(images + static_cast<size_t>(im) * H * H, H, lane, row4, pre);
    const float px_bound = stage_pixels(pre, planes, lane, row4, n_task);
    wave_sync();
    unsigned char* dst = out + static_cast<size_t>(im) * kImgStride;
    for (int i = lane; i < kImgBytes / 16; i += 64)
      reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(planes)[i];
    if (lane == 0) *reinterpret_cast<float*>(dst + kImgBytes) = px_bound;
    wave_sync();
  }
}

template <int NCS, int kConvWaves, bool PRESPLIT>
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
  float* img = lds + kMaxFeat * NCS + wave * kWaveFloats;  // the padded image as two fp16 terms
  float* band = img + kImgBytes / 4;                   // three band buffers of conv1 output
  char* const planes = reinterpret_cast<char*>(img);

  const float* theta = a.params + static_cast<size_t>(member) * a.P;
  const float* W1 = theta;                 // [3][3][1][8]
  const float* b1 = theta + 9 * kC1;       // [8]
  const float* W2 = b1 + kC1;              // [3][3][8][16]
  const float* b2 = W2 + 9 * kC1 * kC2;    // [16]
  const float* Wd = b2 + kC2;              // [n_feat][n_cls]
  const float* bd = Wd + n_feat * n_cls;   // [n_cls]

  // ---- once per workgroup: dense weights -> LDS (rows padded to NCS with zeros) ----------------
  if (n_cls == NCS && (a.P & 1) == 0) {
    // rows of exactly NCS classes: a plain copy, 8 bytes a thread and round, all loads of a thread in flight together
    // (a member's parameter vector is 8-byte aligned when P is even, and Wd starts a multiple of 16 bytes into it);
    // one load per round and iteration took 20 us per workgroup
    constexpr int kRounds = (kMaxFeat * NCS / 2 + 64 * kConvWaves - 1) / (64 * kConvWaves);
    const int n2 = n_feat * NCS / 2;
    float2 v[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int i = threadIdx.x + r * 64 * kConvWaves;
      if (i < n2) v[r] = reinterpret_cast<const float2*>(Wd)[i];
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int i = threadIdx.x + r * 64 * kConvWaves;
      if (i < n2) reinterpret_cast<float2*>(wd_s)[i] = v[r];
    }
  } else {
    for (int i = threadIdx.x; i < n_feat * NCS; i += 64 * kConvWaves) {
      const int f = i / NCS, c = i - f * NCS;
      wd_s[i] = c < n_cls ? Wd[f * n_cls + c] : 0.f;
    }
  }
  // zero the padded buffers once: borders stay zero, interiors are overwritten per image
  for (int i = lane; i < kWaveFloats; i += 64) img[i] = 0.f;

  // conv2 weights as matrix B operands, w2b[output row of the window][term][step]: the step is the tap's column kx,
  // lane group q holds the 8 input channels of band row q, which output row py of the pooling window meets with
  // tap row ky = q - py (zero where that is outside the stencil); column n; each weight split into two terms
  const int n = lane & 15, q = lane >> 4;
  f16x8 w2b[2][2][3];
  float s_w2, u_w2;     // scale of the stored conv2 weights and its reciprocal
  bool lane_bad = false;  // a non-finite convolution weight seen by this lane
  {
    float x[2][3][8];
    float w2_max = 0.f;
#pragma unroll
    for (int py = 0; py < 2; ++py) {
      const int ky = q - py;
#pragma unroll
      for (int st = 0; st < 3; ++st) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          x[py][st][j] = (ky >= 0 && ky < 3) ? W2[((3 * ky + st) * kC1 + j) * kC2 + n] : 0.f;
          w2_max = fmaxf(w2_max, fabsf(x[py][st][j]));
          lane_bad |= !(fabsf(x[py][st][j]) <= kFltMax);
        }
      }
    }
    const float s_w2_ = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(wave_max(w2_max)))));
    s_w2 = s_w2_;
    u_w2 = pow2_reciprocal(s_w2);
#pragma unroll
    for (int py = 0; py < 2; ++py) {
#pragma unroll
      for (int st = 0; st < 3; ++st) {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[py][st][j] *= s_w2_;
        split2_x8_true<true>(x[py][st], w2b[py][0][st], w2b[py][1][st]);
      }
    }
  }
  const float bias2 = b2[n];
  // largest biased exponent of the conv1 activations' scale that keeps |bias2| s_a1 s_w2 below 2^100
  const int e_cap_a1 = __builtin_amdgcn_readfirstlane(
      480 - ((__float_as_int(wave_max(fabsf(bias2))) >> 23) & 0xff) - ((__float_as_int(s_w2) >> 23) & 0xff));
  // the class whose logit this lane ends with (see the reduction after the band loop)
  const int my_cls = 8 * ((lane >> 1) & 1) + 4 * (lane & 1) + 2 * ((lane >> 4) & 1) + ((lane >> 5) & 1);
  const float bias_d = my_cls < n_cls ? bd[my_cls] : 0.f;

  // conv1 weights as matrix A operands.  Row i of the tile is (channel 2 (i >> 2) + (i & 1), pixel column
  // s = (i >> 1) & 1 of the pooling window), so that the four accumulator registers of a lane (rows 4 q .. 4 q + 3
  // of one window) are channels 2 q and 2 q + 1 at both columns.  The contraction runs over the 4 x 4 patch of a
  // window, k = 4 r + c in lane groups 0, 1 (patch rows 0, 1 and 2, 3) against the leading terms of the pixels
  // and again in lane groups 2, 3 against their residual terms; w1a[t] holds the weights shifted to the
  // window's pixel row t (tap (r - t, c - s), zero outside the 3 x 3 stencil).  One instruction with
  // (h | h) and one with (m | 0), m and m' being the residuals themselves, give h h' + m' h + h' m in a single
  // accumulator.  Each
  // channel has its own power of two (its weights' largest magnitude), taken out again by the epilogue.
  f16x8 w1a[2][2];      // [pixel row t][instruction]
  float sw1_row;        // scale of the channel of this lane's A row
  float bound_w1, bound_b1;    // bound on the conv1 activations of any image: max|pixel| * bound_w1 + bound_b1
  {
    const int i = lane & 15, ch = 2 * (i >> 2) + (i & 1), sx = (i >> 1) & 1;
    const int rblk = q & 1, half = q >> 1;
    float wt[9], t_sum = 0.f, t_max = 0.f;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      wt[t] = W1[t * kC1 + ch];
      t_sum += fabsf(wt[t]);
      t_max = fmaxf(t_max, fabsf(wt[t]));
    }
    const float bch = b1[ch];
    lane_bad |= !(t_sum <= kFltMax) || !(fabsf(bch) <= kFltMax) || !(fabsf(bias2) <= kFltMax);
    // at most 2^56, and at most 2^44 / |bias|: with the pixels' scale (at most 2^56, a matter of the image alone) the
    // sums, which start from the scaled bias, then stay below 2^100.  The second limit acts only where a bias is more
    // than 2^29 times its channel's weights.
    sw1_row = __int_as_float(min(min(__float_as_int(split_pow2_scale(t_max)) >> 23, 127 + 56),
                                 297 - ((__float_as_int(bch) >> 23) & 0xff)) << 23);
    bound_w1 = wave_max(t_sum);
    bound_b1 = wave_max(fabsf(bch));
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float x1[8], x2[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int dy = 2 * rblk + (j & 1) - t, dx = (j >> 1) - sx;  // element j: column j >> 1, row j & 1 of the patch rows
        float w = 0.f;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) w = (3 * dy + dx == tap && dx >= 0 && dx <= 2 && dy >= 0 && dy <= 2) ? wt[tap] : w;
        w *= sw1_row;
        const _Float16 h = static_cast<_Float16>(w);
        const float hf = static_cast<float>(h);
        x1[j] = hf;
        x2[j] = half ? 0.f : w - hf;  // the residual, exact in fp32; converted singly below (subnormals kept)
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        w1a[t][0][j] = static_cast<_Float16>(x1[j]);
        w1a[t][1][j] = static_cast<_Float16>(x2[j]);
      }
    }
  }
  // conv1 D role: lane (window n, group q) ends with channels 2 q and 2 q + 1 of its window; their scales come
  // from the lanes whose A rows are those channels (rows 4 q and 4 q + 1)
  float sw1_d[2], b1_d[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    sw1_d[j] = __shfl(sw1_row, 4 * q + j, 64);
    b1_d[j] = b1[2 * q + j];
  }
  // Column n of tile m is the window (pooled row 2 b + (n & 1), column 8 m + (n >> 1)): with both pooled rows of the
  // pass in one tile, the patch reads of 32 lanes and the band stores below fall on different banks.  Patch of
  // that window in the image planes (pass 0): term q >> 1, patch rows 2 (q & 1), 2 (q & 1) + 1.  Its pooled pixel
  // goes to ring row 2 u + 1 + (n & 1) in pass b = 4 k + u (and to the copy of that row where it has one);
  // lane groups 0 and 1 store it (leading and residual term).
  const int n_mt = (H2 + 7) >> 3;   // tiles of 8 window columns x 2 pooled rows per pass
  int p_off[2], own_off[2];
  bool c1_store[2];
  const bool c1_lower = (n & 1) != 0;
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    const int wx = 8 * m + (n >> 1), wxc = min(wx, H2 - 1), rs = n & 1;
    p_off[m] = (q >> 1) * kPlaneBytes + (rs + (q & 1)) * kPairPitch + 8 * wxc;
    own_off[m] = band_off(1 + rs, wxc + 1) + (q & 1) * kBandTerm;  // for u = 0; two rows = one row pair further per u
    c1_store[m] = wx < H2 && q < 2;
  }
  const bool member_bad = __any(lane_bad);

  // conv2 A role of this lane: row r = lane & 15 is the pixel column r of the band (window r >> 1, its column r & 1),
  // lane group q the band's row q: tap column kx reads the pixel kx columns further (the last two rows of the tile
  // belong to a window that no supported image has; their columns are held inside the padded row)
  const int a_off = band_off(q, lane & 15);  // bytes from the first of the band's four ring rows
  char* const bandb = reinterpret_cast<char*>(band);
  // the same as LDS addresses (32-bit), pinned in one register each (the compiler would rather keep the addends
  // apart and add them before every access): what is added per band or per step below is an immediate of the
  // LDS instruction
  typedef __attribute__((address_space(3))) char lds_char;
  auto lds_address = [](const char* p) { return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_char*)p)); };
  auto lds_at = [](uint32_t address, int imm) { return reinterpret_cast<lds_char*>(static_cast<uintptr_t>(address)) + imm; };
  uint32_t a_abs = lds_address(bandb + a_off), own_abs[2], p_abs[2];
  asm volatile("" : "+v"(a_abs));
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    own_abs[h] = lds_address(bandb + own_off[h]);
    p_abs[h] = lds_address(planes + p_off[h]);
    asm volatile("" : "+v"(own_abs[h]));
    asm volatile("" : "+v"(p_abs[h]));
  }
  // the lane's two rows of dense weights in band 0 (windows 2 q and 2 q + 1, channel n)
  uint32_t wr_abs[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    wr_abs[k] = lds_address(reinterpret_cast<const char*>(wd_s + (min(2 * q + k, H4 - 1) * kC2 + n) * NCS));
    asm volatile("" : "+v"(wr_abs[k]));
  }
  // one padded band row (16 pixels of 16 bytes, both terms) set to zero by lanes 0..31
  auto zero_band_row = [&](char* buf, int row) {
    if (lane < 32) *reinterpret_cast<uint4*>(buf + (lane >> 4) * kBandTerm + band_off(row, lane & 15)) = make_uint4(0, 0, 0, 0);
  };

  const int img_begin = blockIdx.x * a.imgs_per_chunk;
  const int img_end = min(a.B, img_begin + a.imgs_per_chunk);
  const int row4 = H / 4, n_task = (H / 2 + 1) * row4;  // float4 pieces of a row; (row pair, piece) tasks of an image
  float loss_sum = 0.f;

  // prefetch of the first image: lane takes pieces lane, lane + 64, ... (of its pixels, or of its split planes)
  float4 pre[4] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f),
                   make_float4(0.f, 0.f, 0.f, 0.f)};  // pieces beyond the image stay zero
  uint4 pre_split[4] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
  auto prefetch = [&](int image) {
    if (PRESPLIT) {
      const uint4* src = reinterpret_cast<const uint4*>(a.planes + static_cast<size_t>(image) * kImgStride);
#pragma unroll
      for (int j = 0; j < 4; ++j) pre_split[j] = src[lane + 64 * j];  // kImgStride = 4 x 64 x 16 bytes
    } else {
      load_pixels(a.images + static_cast<size_t>(image) * H * H, H, lane, row4, pre);
    }
  };
  int im = img_begin + wave;
  if (im < img_end) prefetch(im);
  __syncthreads();  // dense weights staged

  for (; im < img_end; im += kConvWaves) {
    // ---- the image as two fp16 terms in the zero-padded planes (split here, or copied from the batch split once
    //      for all members); then prefetch the next image -------
    float px_bound;
    if (PRESPLIT) {
      static_assert(kImgBytes == 3 * 1024 + 48 * 16 && kImgStride == 4096, "three full rounds of 16 bytes a lane and 48 lanes of a fourth");
#pragma unroll
      for (int j = 0; j < 3; ++j) *reinterpret_cast<uint4*>(planes + 16 * (lane + 64 * j)) = pre_split[j];
      if (lane < 48) *reinterpret_cast<uint4*>(planes + 16 * (lane + 192)) = pre_split[3];
      px_bound = __uint_as_float(__builtin_amdgcn_readlane(pre_split[3].x, 48));  // the float behind the planes
    } else {
      px_bound = stage_pixels(pre, planes, lane, row4, n_task);
    }
    // scales of this image (all wave-uniform): of its pixels from their largest magnitude, of its conv1 activations
    // from the bound on them
    const float a1_bound = fmaf(px_bound, bound_w1, bound_b1);
    // (limited so that the conv2 sums, which start from the scaled bias, stay below 2^100: the limit acts only where a
    // conv2 bias is more than 2^70 times the convolution it is added to)
    const float s_a1 = __int_as_float(__builtin_amdgcn_readfirstlane(
        min(__float_as_int(split_pow2_scale(a1_bound)) >> 23, e_cap_a1) << 23));
    const float u_a2 = pow2_reciprocal(s_a1) * u_w2;
    // the conv2 bias in the units of the conv2 sums (the smaller factor first: no intermediate overflow)
    const float bias2_init = (bias2 * fminf(s_a1, s_w2)) * fmaxf(s_a1, s_w2);
    const bool image_bad = member_bad || !(a1_bound <= kFltMax);
    const float s_px = pixel_scale(px_bound);
    float c1_init[2], c1_out[2];  // accumulators start from the scaled bias; factor from them to the stored activations
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float both = sw1_d[j] * s_px;
      c1_init[j] = b1_d[j] * both;
      c1_out[j] = s_a1 * pow2_reciprocal(both);
    }
    if (im + kConvWaves < img_end) prefetch(im + kConvWaves);
    wave_sync();

    float acc[NCS];  // the dense layer's partial sums of this lane, per class
#pragma unroll
    for (int c = 0; c < NCS; ++c) acc[c] = 0.f;
    // conv2 D role: the registers of lane (q, n) are the two pixel columns of windows 2 q and 2 q + 1 of channel n,
    // one accumulator per pixel row: two features of the dense layer, which is accumulated band by band (per lane
    // and class) from the workgroup's copy of its weights.
    const float u_win[2] = {2 * q < H4 ? u_a2 : 0.f, 2 * q + 1 < H4 ? u_a2 : 0.f};  // zero: a window beyond the image
    const int dense_band_bytes = H4 * kC2 * NCS * 4;  // dense weights of one band of features
    auto dense_of_band = [&](const floatx4 (&sums)[2], int bd) {
      // ReLU of the largest of four, on the bit patterns as for conv1 (the sums carry the bias already); the factor
      // to true units, a power of two, comes after
      const int m0 = max(max(max(__float_as_int(sums[0][0]), __float_as_int(sums[0][1])),
                             max(__float_as_int(sums[1][0]), __float_as_int(sums[1][1]))), 0);
      const int m1 = max(max(max(__float_as_int(sums[0][2]), __float_as_int(sums[0][3])),
                             max(__float_as_int(sums[1][2]), __float_as_int(sums[1][3]))), 0);
      const float x0 = __int_as_float(m0) * u_win[0], x1 = __int_as_float(m1) * u_win[1];
      typedef __attribute__((address_space(3))) const f32x2 lds_f32x2;  // rows of NCS floats: 8-byte aligned
      const uint32_t band_bytes = static_cast<uint32_t>(bd * dense_band_bytes);
      const uint32_t wr0 = wr_abs[0] + band_bytes, wr1 = wr_abs[1] + band_bytes;
#pragma unroll
      for (int c = 0; c < NCS; c += 2) {
        const f32x2 w0 = *reinterpret_cast<lds_f32x2*>(lds_at(wr0, 4 * c));
        const f32x2 w1 = *reinterpret_cast<lds_f32x2*>(lds_at(wr1, 4 * c));
        acc[c] = fmaf(x1, w1[0], fmaf(x0, w0[0], acc[c]));
        acc[c + 1] = fmaf(x1, w1[1], fmaf(x0, w0[1], acc[c + 1]));
      }
    };
    zero_band_row(bandb, 0);  // ring row 0: the border above the image
    // Four passes per round of the ring, written out so that every ring address is a lane constant plus an
    // immediate: pass b = b0 + u stores to ring rows 2 u + 1, 2 u + 2, the conv2 band behind it starts at row
    // 2 ((u + 3) & 3).
#pragma unroll 1
    for (int b0 = 0; b0 <= H4; b0 += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = b0 + u;
      if (b > H4) break;
      // ---- conv1 + ReLU + pool, pass b: pooled rows 2b and 2b+1 ----
      if (b == H4) {
        zero_band_row(bandb, 2 * ((H4 - 1) & 3) + 3);  // the border below the image: last row of the last band
      } else {
        // the tiles of the pass side by side, stage by stage (reads, matrix instructions, pooling, stores), so that
        // the dependent chain of one tile runs in the gaps of the other's
        auto conv1_pass = [&](auto tiles) {
          constexpr int NM = decltype(tiles)::value;
          const floatx4 c_init = {c1_init[0], c1_init[1], c1_init[0], c1_init[1]};
          typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));
          f16x8 patch[NM];
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            // the lane's eight patch values: four consecutive columns of a row pair
            typedef uint32_t u32x2p __attribute__((ext_vector_type(2)));
            typedef __attribute__((address_space(3))) const u32x2p lds_u2;  // 8-byte aligned: one ds_read2_b64
            const lds_char* pp = lds_at(p_abs[m] + b0 * (2 * kPairPitch), u * (2 * kPairPitch));
            const u32x2p lo = *reinterpret_cast<lds_u2*>(pp), hi = *reinterpret_cast<lds_u2*>(pp + 8);
            const u32x4p pw = {lo[0], lo[1], hi[0], hi[1]};
            patch[m] = __builtin_bit_cast(f16x8, pw);
          }
          floatx4 o0[NM], o1[NM];
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            o0[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1a[0][0], patch[m], c_init, 0, 0, 0);
            o1[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1a[1][0], patch[m], c_init, 0, 0, 0);
          }
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            o0[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1a[0][1], patch[m], o0[m], 0, 0, 0);
            o1[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1a[1][1], patch[m], o1[m], 0, 0, 0);
          }
          u32x4p pixel[NM];
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            // pooling window of channels 2 q, 2 q + 1: both pixel rows (o0, o1) and both columns (registers i, i + 2).
            // ReLU of the largest of four = the largest of the four and zero, taken on the bit patterns as signed
            // integers: among non-negative floats they order like the floats, and every negative float (and -0) is a
            // negative integer, which the zero beats.  The factor to the stored units (a power of two) comes after.
            const float r0 = __int_as_float(max(max(max(__float_as_int(o0[m][0]), __float_as_int(o0[m][2])),
                                                    max(__float_as_int(o1[m][0]), __float_as_int(o1[m][2]))), 0));
            const float r1 = __int_as_float(max(max(max(__float_as_int(o0[m][1]), __float_as_int(o0[m][3])),
                                                    max(__float_as_int(o1[m][1]), __float_as_int(o1[m][3]))), 0));
            uint32_t lead, resid;
            split2_pair_true(r0 * c1_out[0], r1 * c1_out[1], lead, resid);
            // the four channel pairs of a window (lane groups 0..3) -> the 16 bytes of its pixel, leading term in
            // lane group 0 and residual term in lane group 1: one swap between neighbouring groups, then the
            // upper half of the wave moves down (what the swaps leave in the upper half is not stored; their second
            // operands are values that are dead by now, so no copies are made to preserve them)
            const auto sw = __builtin_amdgcn_permlane16_swap(lead, resid, false, false);   // (L0 R0 L2 R2), (L1 R1 L3 R3)
            const auto s2 = __builtin_amdgcn_permlane32_swap(sw[0], __float_as_uint(o0[m][0]), false, false);  // groups 0, 1: own, then L2, R2
            const auto s3 = __builtin_amdgcn_permlane32_swap(sw[1], __float_as_uint(o1[m][0]), false, false);  // groups 0, 1: own, then L3, R3
            pixel[m] = u32x4p{s2[0], s3[0], s2[1], s3[1]};
          }
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            if (c1_store[m]) {
              typedef __attribute__((address_space(3))) u32x4p lds_u4;
              *reinterpret_cast<lds_u4*>(lds_at(own_abs[m], u * kBandRowPair)) = pixel[m];
              // ring rows 1 and 8 have a copy (rows 9 and 0)
              if (u == 0 && !c1_lower) *reinterpret_cast<lds_u4*>(lds_at(own_abs[m], 4 * kBandRowPair)) = pixel[m];
              if (u == 3 && c1_lower) *reinterpret_cast<lds_u4*>(lds_at(own_abs[m], -kBandRowPair)) = pixel[m];
            }
          }
        };
        if (n_mt == 2) conv1_pass(std::integral_constant<int, 2>());
        else conv1_pass(std::integral_constant<int, 1>());
      }
      wave_sync();
      if (b == 0) continue;

      // ---- conv2 + ReLU + pool, band b-1: one tile of all its pixel columns, one accumulator per output row ----
      const int bb = ((u + 3) & 3) * kBandRowPair;  // bytes from ring row 0 to the band's first row
      const floatx4 c2_init = {bias2_init, bias2_init, bias2_init, bias2_init};
      floatx4 accp[2] = {c2_init, c2_init};  // bias + h h' + h m' + m h' (residual terms unscaled)
      // One 16-byte read per split term: the lane's pixel (band row q, column r).  Tap columns 1 and 2 are the pixels
      // of the lanes one and two columns further in the same lane group (row_shl moves; the last lanes of a group,
      // which get zeros, belong to the window that does not exist).
      f16x8 at[2][3];  // [term][tap column]
      typedef __attribute__((address_space(3))) const f16x8 lds_f16x8;
      typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        at[k][0] = *reinterpret_cast<lds_f16x8*>(lds_at(a_abs, bb + k * kBandTerm));
        const u32x4s w = __builtin_bit_cast(u32x4s, at[k][0]);
        u32x4s w1, w2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          w1[i] = __builtin_amdgcn_update_dpp(0, w[i], 0x101, 0xf, 0xf, true);  // row_shl:1
          w2[i] = __builtin_amdgcn_update_dpp(0, w[i], 0x102, 0xf, 0xf, true);  // row_shl:2
        }
        at[k][1] = __builtin_bit_cast(f16x8, w1);
        at[k][2] = __builtin_bit_cast(f16x8, w2);
      }
#pragma unroll
      for (int st = 0; st < 3; ++st) {
#pragma unroll
        for (int py = 0; py < 2; ++py) accp[py] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at[1][st], w2b[py][0][st], accp[py], 0, 0, 0);
#pragma unroll
        for (int py = 0; py < 2; ++py) accp[py] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at[0][st], w2b[py][1][st], accp[py], 0, 0, 0);
#pragma unroll
        for (int py = 0; py < 2; ++py) accp[py] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at[0][st], w2b[py][0][st], accp[py], 0, 0, 0);
      }
      // the band before this one, whose sums were carried over: independent of the matrix instructions above,
      // so its vector work can be issued between them
      dense_of_band(accp, b - 1);
      wave_sync();
    }
    }


    // Sum over the 64 lanes, per class, in registers: every step adds the two halves of a lane pairing and halves
    // the number of live classes, the lanes of one half keeping the even and the others the odd ones.  Halves of
    // the wave and neighbouring rows first (a swap and an add per pair of classes), then lanes 1 and 2 apart; the
    // quads of a row then hold copies, which one rotation by four and one by eight add up.  Lane l ends with the
    // class 8 b1 + 4 b0 + 2 b4 + b5 of its bits (my_cls).
    float logit;
    {
      constexpr int N1 = (NCS + 1) / 2, N2 = (N1 + 1) / 2, N3 = (N2 + 1) / 2;
      static_assert(NCS % 2 == 0 && NCS <= 16 && NCS > 8, "class counts this reduction is written for");
      float w[N1], x[N2], y[N3];
#pragma unroll
      for (int j = 0; j < N1; ++j) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[2 * j]), __float_as_uint(acc[2 * j + 1]), false, false);
        w[j] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
      }
#pragma unroll
      for (int k = 0; k < N2; ++k) {
        const uint32_t other = 2 * k + 1 < N1 ? __float_as_uint(w[2 * k + 1 < N1 ? 2 * k + 1 : 0]) : 0u;
        const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(w[2 * k]), other, false, false);
        x[k] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
      }
      const bool odd1 = (lane & 1) != 0, odd2 = (lane & 2) != 0;
#pragma unroll
      for (int m = 0; m < N3; ++m) {
        if (2 * m + 1 < N2) {
          const float keep = odd1 ? x[2 * m + 1 < N2 ? 2 * m + 1 : 0] : x[2 * m];
          const float send = odd1 ? x[2 * m] : x[2 * m + 1 < N2 ? 2 * m + 1 : 0];
          y[m] = keep + dpp_mov<0xB1>(send);
        } else {
          const float both = x[2 * m] + dpp_mov<0xB1>(x[2 * m]);
          y[m] = odd1 ? 0.f : both;
        }
      }
      static_assert(N3 == 2, "two registers left before the last halving");
      {
        const float keep = odd2 ? y[1] : y[0], send = odd2 ? y[0] : y[1];
        logit = keep + dpp_mov<0x4E>(send);
      }
      logit += dpp_mov<0x124>(logit);  // row_ror:4
      logit += dpp_mov<0x128>(logit);  // row_ror:8
      logit += bias_d;
    }
    if (image_bad) logit = __builtin_nanf("");  // a non-finite weight or pixel: what fp32 arithmetic would propagate

    if (a.out) {
      if ((lane & 12) == 0 && my_cls < n_cls)
        a.out[(static_cast<size_t>(member) * a.B + im) * n_cls + my_cls] = logit;
    } else {
      // cross-entropy over the classes (those beyond n_cls count as -inf): the last quad of every row holds four
      // of them, so a reduction runs over the quad and then down the rows into lane 63
      const int y = a.labels[im];  // a label outside [0, n_cls) contributes logit 0
      const float lv = my_cls < n_cls ? logit : -INFINITY;
      const float mx = last_lane(quads_max(lv));
      // the hardware's exp2 and log2 (one ulp each): the terms are at most one and their sum lies in [1, 16]
      const float se = last_lane(quads_sum(my_cls < n_cls ? __builtin_amdgcn_exp2f(1.4426950408889634f * (lv - mx)) : 0.f));
      const float picked = last_lane(quads_sum(my_cls == y ? lv : 0.f));
      loss_sum += (mx + 0.6931471805599453f * __builtin_amdgcn_logf(se)) - picked;
    }
    wave_sync();
  }

  if (a.partial) {
    if (lane == 0) wave_loss[wave] = loss_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.f;
      for (int w = 0; w < kConvWaves; ++w) t += wave_loss[w];
      if (a.fitness) a.fitness[member] = a.scale * t;
      else a.partial[static_cast<size_t>(member) * a.chunks + blockIdx.x] = t;
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

// Workgroups per member: the count that minimises (rounds of the grid over the chip's 256 compute units, one
// workgroup each) x (a workgroup's set-up, measured at about 25 images' worth, + its images, in rounds of one image
// per wave); no fewer than one image per wave.  cfg2 (256 members, 1024 images): one workgroup per member.
int convnet_chunks(const ConvShape&, int pop, int B) {
  constexpr int kCUs = 256, kSetupImages = 25;
  const int max_chunks = max(1, min((B + kConvWavesMax - 1) / kConvWavesMax, 64));
  int best = 1;
  long best_cost = -1;
  for (int c = 1; c <= max_chunks; ++c) {
    const long rounds = (static_cast<long>(pop) * c + kCUs - 1) / kCUs;
    const int images = (B + c - 1) / c;
    const long per_group = kSetupImages + kConvWavesMax * ((images + kConvWavesMax - 1) / kConvWavesMax);
    const long cost = rounds * per_group;
    if (best_cost < 0 || cost < best_cost) best = c, best_cost = cost;
  }
  return best;
}

template <int NCS, int WAVES, bool PRESPLIT>
static int launch_conv(const ConvArgs& a, int pop, hipStream_t s) {
  const size_t shmem = sizeof(float) * (static_cast<size_t>(kMaxFeat) * NCS + WAVES * kWaveFloats);
  static_assert(sizeof(float) * (kMaxFeat * NCS + WAVES * kWaveFloats) + 256 <= 160 * 1024, "LDS budget of a CU");
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(convnet_kernel<NCS, WAVES, PRESPLIT>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
  if (e != hipSuccess) (void)hipGetLastError();  // do not leave the error sticky for the caller's next HIP call
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((convnet_kernel<NCS, WAVES, PRESPLIT>), dim3(a.chunks, pop), dim3(64 * WAVES), shmem, s, a);
  return check_launch("convnet_kernel");
}

// Bytes of workspace for the batch split once for all members.
size_t convnet_planes_bytes(int B) { return static_cast<size_t>(B) * kImgStride; }

int launch_convnet_f32(const ConvShape& sh, const float* params, const float* images, int pop, int B, float* out,
                       const int32_t* labels, float* partial, int chunks, void* planes_work, float* fitness, float scale,
                       hipStream_t s) {
  ConvArgs a;
  a.params = params, a.images = images, a.labels = labels, a.out = out, a.partial = partial;
  a.planes = static_cast<const unsigned char*>(planes_work);
  a.P = sh.P, a.H = sh.H, a.n_cls = sh.n_cls, a.B = B;
  if (chunks <= 0) chunks = convnet_chunks(sh, pop, B);
  a.chunks = chunks;
  a.imgs_per_chunk = (B + chunks - 1) / chunks;
  a.fitness = chunks == 1 ? fitness : nullptr, a.scale = scale;
  if (planes_work) {
    // the split of the batch into fp16 terms is the same for every member: done once, ahead of the members' kernel
    const int blocks = min((B + kSplitWaves - 1) / kSplitWaves, 1024);
    hipLaunchKernelGGL(convnet_split_kernel, dim3(blocks), dim3(64 * kSplitWaves), 0, s, images, B, sh.H,
                       static_cast<unsigned char*>(planes_work));
    const int rc = check_launch("convnet_split_kernel");
    if (rc) return rc;
    return sh.n_cls == 10 ? launch_conv<10, 12, true>(a, pop, s) : launch_conv<16, 10, true>(a, pop, s);
  }
  return sh.n_cls == 10 ? launch_conv<10, 12, false>(a, pop, s) : launch_conv<16, 10, false>(a, pop, s);
}

}  // namespace evo
