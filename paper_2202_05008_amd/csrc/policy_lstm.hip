// A policy with carried state: the LSTM sequence-to-sequence model of the paper's "Seq2Seq
// Learning" example (Section 3: the query is the string of an addition, "012+345=", the answer the
// string of the sum) evaluated for every member with its own weights on one shared batch; the
// cells (h, c) are the policy state that Section 4 ("Exploring Novel Policy Architectures")
// passes from one get_actions call to the next.  Here the whole sequence runs inside one kernel
// and that state never leaves the chip.
//
// Model.  Tokens are integers below V; an encoder cell reads the query, a decoder cell (own weights)
// starts from the encoder's final (h, c) and takes one step per answer position, fed with the token
// '=' (V - 1) first and with the true previous answer digit afterwards; logits_j = h_j Wo + bo.
//   a = Wx[token] + h Wh + b   (gates i, f, g, o: columns g H + u)
//   c' = sigmoid(a_f) c + sigmoid(a_i) tanh(a_g);   h' = sigmoid(a_o) tanh(c')
// Flat parameters: enc Wx[V][4H], Wh[H][4H], b[4H]; dec Wx, Wh, b; Wo[H][n_out]; bo[n_out].
//
// Mapping.  One workgroup owns one member; wave w owns hidden units 16 w .. 16 w + 15 in all four
// gates, and the 64 K recurrent weights of the active cell sit in the registers of the workgroup's
// waves as matrix-core operands for the whole phase (H = 128: 128 registers per lane).  The
// recurrent product runs transposed on v_mfma_f32_16x16x32_f16: rows = the wave's 16 units of one
// gate, columns = 16 samples, so that a lane ends up with the four gates of four consecutive units
// of one sample: the cell update is lane-local, c stays in registers, and h' leaves as one 8-byte
// LDS store per split term.  h is kept in LDS as two half-precision terms (split16.h: 22
// significand bits, three matrix instructions per product into one accumulator, within a few 1e-7 of
// fp32 arithmetic).
// h lies in (-1, 1) and is stored times 2^14; the recurrent weights of a wave are stored times a power
// of two s_w, so the gate pre-activations come out times 2^14 s_w and the factor is folded into the
// exp2 arguments of the sigmoids and tanh.  The kernel is built twice.  The first build takes s_w = 2^12,
// which holds every weight below 15.99 (and keeps the residual term of every weight above 2^-15 a normal number), checks the weights as it loads them, and marks a member that has a
// larger one (its result is a NaN with a payload of its own).  The second build is launched right behind
// it over the same grid: a workgroup whose member is not marked exits at once; for a marked member each
// wave first reads its weights once more to find their largest magnitude and scales them by the power of
// two that fits it, so any finite weight is representable.  Members in range pay one empty workgroup.
// (The output layer, being small, always takes its scale from its largest weight.)
// The input term needs no product at all: a
// one-hot token selects a row of Wx, which is kept with the bias added in an LDS table.  A step
// writes h' into a buffer nobody reads, so one workgroup barrier per step suffices.  Samples are
// processed in chunks of 64 (four column tiles); two chunks are in flight per pass (three h
// buffers rotate: the current h of each chunk and the free one), so that a cell's weights are
// loaded once per 128 samples.  The weights arrive with coalesced 16-byte loads that are all in
// flight together and reach their owners through LDS.
//
// Register layouts (lane = 16 q + j):  A[row j][k = 8 q + e], B[k = 8 q + e][col j], e = 0..7;
// D[row 4 q + i][col j], i = 0..3.
#include "kernels.h"
#include "split16.h"

namespace evo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kChunk = 64;            // samples per pass: four column tiles
constexpr int kMaxV = 16, kMaxOut = 16, kMaxLq = 32, kMaxLa = 16;
constexpr float kSH = 16384.0f;                 // 2^14: scale of the stored h
constexpr float kSWDefault = 4096.0f;           // 2^12: scale of the stored weights unless one of them would overflow
constexpr float kSplitMax = 65504.0f;           // largest finite fp16
constexpr uint32_t kMarkBits = 0x7fc5eed5u;     // the quiet NaN that marks a member for the second build
constexpr float kLog2e = 1.4426950408889634f;

// sigmoid and tanh of a pre-activation that is held times 1 / u (k = log2(e) u rides in the exp2 argument)
__device__ __forceinline__ float exp_neg_scaled(float A, float k) { return __builtin_amdgcn_exp2f((-k) * A); }
__device__ __forceinline__ float sigmoid_scaled(float A, float k) {
  return __builtin_amdgcn_rcpf(1.0f + exp_neg_scaled(A, k));
}
__device__ __forceinline__ float tanh_scaled(float A, float k) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f((2.0f * k) * A) + 1.0f);
}

__device__ __forceinline__ float tanh_fast(float x) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f((2.0f * kLog2e) * x) + 1.0f);
}

struct LstmArgs {
  const float* params;
  const int32_t* query;   // [B][Lq]
  const int32_t* answer;  // [B][La]
  float* fitness;         // [pop] or null
  float* logits;          // [pop][B][La][n_out] or null
  int P, B, Lq, La, V, n_out;
};

// One cell step of one chunk of 64 samples: gates from the current h (LDS, two terms), cell
// update in registers, h' into the free buffer.  `tok_of(s)` gives the input token of sample s.
template <int H, typename TokOf>
__device__ __forceinline__ void lstm_step(const f16x8 (&wh)[2][4][H / 32], floatx4 (&cst)[4], const float* tab,
                                          const unsigned char* hc, unsigned char* hn, int wave, int j, int q,
                                          float k_u, TokOf tok_of) {
  constexpr int KS = H / 32, kRowB = (H + 8) * 2, kTermB = kChunk * kRowB, kTabRow = 4 * H + 4;
#pragma unroll
  for (int st = 0; st < 4; ++st) {
    const int s = 16 * st + j;  // this lane's sample (column)
    const int tok = tok_of(s);
    floatx4 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      acc[g] = *reinterpret_cast<const floatx4*>(tab + tok * kTabRow + g * H + 16 * wave + 4 * q);
    const unsigned char* src = hc + s * kRowB + 16 * q;
#pragma unroll
    for (int kb = 0; kb < KS; ++kb) {
      const f16x8 b0 = *reinterpret_cast<const f16x8*>(src + 64 * kb);
      const f16x8 b1 = *reinterpret_cast<const f16x8*>(src + kTermB + 64 * kb);
      // three rounds over the gates (four independent instructions between two that share an accumulator), the
      // small partial products first
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wh[0][g][kb], b1, acc[g], 0, 0, 0);
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wh[1][g][kb], b0, acc[g], 0, 0, 0);
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wh[0][g][kb], b0, acc[g], 0, 0, 0);
    }
    // ---- cell update of units 16 wave + 4 q + i for sample s; h' (times 2^14) -> the free buffer ----
    float hs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float ai = acc[0][i], af = acc[1][i], ag = acc[2][i], ao = acc[3][i];
      const float c = fmaf(sigmoid_scaled(af, k_u), cst[st][i], sigmoid_scaled(ai, k_u) * tanh_scaled(ag, k_u));
      cst[st][i] = c;
      // 2^14 sigmoid(a_o) = 1 / (2^-14 (1 + e^-a_o))
      const float so = __builtin_amdgcn_rcpf(fmaf(exp_neg_scaled(ao, k_u), 1.0f / kSH, 1.0f / kSH));
      hs[i] = so * tanh_fast(c);
    }
    uint2 lead, resid;
    split2_pair_true(hs[0], hs[1], lead.x, resid.x);
    split2_pair_true(hs[2], hs[3], lead.y, resid.y);
    unsigned char* dst = hn + s * kRowB + (16 * wave + 4 * q) * 2;
    *reinterpret_cast<uint2*>(dst) = lead;
    *reinterpret_cast<uint2*>(dst + kTermB) = resid;
  }
}

}  // namespace

// DYNAMIC: the second build (see the head of the file).
template <int H, bool DYNAMIC>
__global__ __launch_bounds__(4 * H) void lstm_seq2seq_kernel(LstmArgs a) {
  constexpr int NW = H / 16;            // waves
  constexpr int KS = H / 32;            // matrix-core steps over the hidden units
  constexpr int G4 = 4 * H;             // gate columns
  constexpr int kRowB = (H + 8) * 2;    // bytes of one sample's row of one term (16 bytes of padding)
  constexpr int kTermB = kChunk * kRowB;
  constexpr int kBufB = 2 * kTermB;     // both terms of one h buffer
  constexpr int kTabRow = G4 + 4;       // floats per token row: 16 bytes of padding spread the tokens over the banks
  // three h buffers: the current h of each of the two chunks in flight and the one the next step writes
  __shared__ __attribute__((aligned(16))) unsigned char hbuf[3 * kBufB];
  __shared__ __attribute__((aligned(16))) float tab[kMaxV * kTabRow];     // 2^14 s_w (Wx[token] + b) of the active cell
  __shared__ __attribute__((aligned(16))) f16x8 wo_s[2][KS][64];          // Wo^T as A operands, two terms
  __shared__ unsigned char tokq[2 * kChunk * kMaxLq];
  __shared__ unsigned char toka[2 * kChunk * kMaxLa];
  __shared__ float wave_loss[NW];
  __shared__ float wave_scale[NW];  // 2^14 s_w of each wave's columns of the active cell (for the input table)
  __shared__ float wg_max[NW];
  __shared__ int refetch;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, q = lane >> 4;
  const int member = blockIdx.x;
  const int V = a.V, n_out = a.n_out, Lq = a.Lq, La = a.La;
  const float* theta = a.params + static_cast<size_t>(member) * a.P;
  const int cell_size = V * G4 + H * G4 + G4;
  const float* Wo = theta + 2 * cell_size;
  const float* bo = Wo + H * n_out;
  // where the mark of this member lives: its fitness, or else its first logit
  float* const mark = a.fitness ? a.fitness + member
                                : a.logits + static_cast<size_t>(member) * a.B * La * n_out;
  if (DYNAMIC) {
    if (tid == 0) refetch = __float_as_uint(*mark) == kMarkBits;
    __syncthreads();
    if (!refetch) return;
  }
  float range_max = 0.f;  // first build: largest |weight| this thread has seen

  // ---- once: output layer as A operands (row j = output j, zero beyond n_out), scaled by the power of two that
  //      fits its largest weight; bias of this lane's rows ----
  float u_o;  // 1 / (2^14 s_o)
  {
    float m = 0.f;
    for (int i = tid; i < H * n_out; i += 4 * H) m = fmaxf(m, fabsf(Wo[i]));
    m = wave_max(m);
    if (lane == 0) wg_max[wave] = m;
    __syncthreads();
    m = wg_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, wg_max[w]);
    const float s_o = split_pow2_scale(m);
    u_o = pow2_reciprocal(s_o) * (1.0f / kSH);
    for (int i = tid; i < KS * 64; i += 4 * H) {
      const int kb = i >> 6, l = i & 63, jj = l & 15, qq = l >> 4;
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = jj < n_out ? s_o * Wo[(32 * kb + 8 * qq + e) * n_out + jj] : 0.f;
      split2_x8_true<true>(x, wo_s[0][kb][l], wo_s[1][kb][l]);
    }
  }
  float bo4[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bo4[i] = 4 * q + i < n_out ? bo[4 * q + i] : 0.f;

  float loss_acc = 0.f;  // sum over this lane's samples and positions (lanes with q == 0 of waves 0..3)

  // Byte offsets of this thread's four 16-byte pieces inside a 16-row piece of a recurrent matrix:
  // float4 f = tid + 4 H i sits in row r = f / H (matrix row 8 (r >> 2) + (r & 3) of the piece), column 4 (f % H).
  uint32_t lane_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int f = tid + 4 * H * i, r = f / H, c4 = f - r * H;
    lane_off[i] = static_cast<uint32_t>(((8 * (r >> 2) + (r & 3)) * G4 + 4 * c4) * 4);
  }

  // Two chunks of 64 samples share one load of each cell's weights.
  for (int c0 = 0; c0 < a.B; c0 += 2 * kChunk) {
    const int n_chunks = a.B - c0 > kChunk ? 2 : 1;
    // ---- tokens -> LDS (samples beyond B read token 0 and are masked from the loss) ----
    __syncthreads();  // the previous pass is done with the token arrays and the h buffers
    for (int i = tid; i < 2 * kChunk * Lq; i += 4 * H) {
      const int s = i / Lq, t = i - s * Lq;
      const int v = c0 + s < a.B ? a.query[static_cast<size_t>(c0 + s) * Lq + t] : 0;
      tokq[s * kMaxLq + t] = static_cast<unsigned char>(min(max(v, 0), V - 1));
    }
    for (int i = tid; i < 2 * kChunk * La; i += 4 * H) {
      const int s = i / La, t = i - s * La;
      const int v = c0 + s < a.B ? a.answer[static_cast<size_t>(c0 + s) * La + t] : 0;
      toka[s * kMaxLa + t] = static_cast<unsigned char>(min(max(v, 0), n_out - 1));
    }
    for (int i = tid; i < 2 * kBufB / 4; i += 4 * H) reinterpret_cast<uint32_t*>(hbuf)[i] = 0u;  // h_0 = 0, both chunks
    floatx4 cst[2][4];  // c of (chunk, units 16 wave + 4 q + i, sample 16 st + j)
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
      for (int st = 0; st < 4; ++st) cst[ch][st] = floatx4{0.f, 0.f, 0.f, 0.f};
    int cur0 = 0, cur1 = 1, spare = 2;  // buffers holding h of chunk 0, of chunk 1, and the free one

#pragma unroll 1
    for (int phase = 0; phase < 2; ++phase) {
      const float* Wx = theta + phase * cell_size;
      const float* Wh = Wx + V * G4;
      const float* bg = Wh + H * G4;
      // ---- recurrent weights of this cell -> registers: wh[term][gate][step], element e is
      //      s_w Wh[32 step + 8 q + e][gate H + 16 wave + j].  The whole matrix is fetched with 16-byte
      //      loads that are all in flight at once (one round trip to memory per cell), then handed
      //      through LDS in pieces of 16 rows (the area of the token table, free between two cells):
      //      piece (step, half) holds rows 32 step + 8 q' + 4 half + e', q' = 0..3, e' = 0..3. ----
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      constexpr int kPieces = 2 * KS;            // 16 rows each
      constexpr int kVecPerThread = 4;           // float4 per thread and piece: 16 rows x H float4 over 4 H threads
      constexpr int kBatch = kPieces < 4 ? kPieces : 4;  // pieces fetched together (64 registers of raw weights)
      f16x8 wh[2][4][KS];
      float s_w = kSWDefault;  // scale of this wave's weights (wave-uniform)
      if (DYNAMIC) {
        // the wave's own columns (gate g, unit 16 wave + j), all rows: their largest magnitude sets the scale
        float w_max = 0.f;
        for (int k = q; k < H; k += 4)
#pragma unroll
          for (int g = 0; g < 4; ++g) w_max = fmaxf(w_max, fabsf(Wh[k * G4 + g * H + 16 * wave + j]));
        s_w = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(split_pow2_scale(wave_max(w_max)))));
      }
#pragma unroll
      for (int p0 = 0; p0 < kPieces; p0 += kBatch) {
        f32x4 raw[kBatch][kVecPerThread];
#pragma unroll
        for (int pb = 0; pb < kBatch; ++pb) {
          const int pc = p0 + pb;
          // uniform base of the piece + four per-lane byte offsets that are the same for every piece
          const char* piece = reinterpret_cast<const char*>(Wh + (32 * (pc >> 1) + 4 * (pc & 1)) * G4);
#pragma unroll
          for (int i = 0; i < kVecPerThread; ++i) raw[pb][i] = *reinterpret_cast<const f32x4*>(piece + lane_off[i]);
        }
#pragma unroll
        for (int pb = 0; pb < kBatch; ++pb) {
          const int pc = p0 + pb;
          __syncthreads();  // the table (or the previous piece) is no longer read
#pragma unroll
          for (int i = 0; i < kVecPerThread; ++i) {
            const int f = tid + 4 * H * i;
            const int r = f / H, c4 = f - r * H;
            *reinterpret_cast<f32x4*>(tab + r * kTabRow + 4 * c4) = raw[pb][i];
          }
          __syncthreads();
          float x[4][4];
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              x[g][e] = s_w * tab[(4 * q + e) * kTabRow + g * H + 16 * wave + j];
              if (!DYNAMIC) range_max = fmaxf(range_max, fabsf(x[g][e]));
            }
          // rows e = 0..3 (4..7) of the step are the first (second) two words of the operands: split as they arrive.
          // The second build's weights may lie far below their wave's largest one: their residuals are kept.
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            u32x4 l = __builtin_bit_cast(u32x4, wh[0][g][pc >> 1]), r = __builtin_bit_cast(u32x4, wh[1][g][pc >> 1]);
#pragma unroll
            for (int w = 0; w < 2; ++w) {
              uint32_t lw, rw;
              if (DYNAMIC) split2_pair_true_kept(x[g][2 * w], x[g][2 * w + 1], lw, rw);
              else split2_pair_true(x[g][2 * w], x[g][2 * w + 1], lw, rw);
              l[2 * (pc & 1) + w] = lw;
              r[2 * (pc & 1) + w] = rw;
            }
            wh[0][g][pc >> 1] = __builtin_bit_cast(f16x8, l);
            wh[1][g][pc >> 1] = __builtin_bit_cast(f16x8, r);
          }
        }
        __builtin_amdgcn_sched_barrier(0);  // the next batch is fetched only now: its registers are the ones just freed
      }
      const float k_u = kLog2e * (pow2_reciprocal(s_w) * (1.0f / kSH));  // log2(e) / (2^14 s_w)
      if (DYNAMIC && lane == 0) wave_scale[wave] = kSH * s_w;
      __syncthreads();  // every wave has read the last piece
      for (int i = tid; i < V * G4; i += 4 * H) {
        const int col = i % G4;
        // in the units of its wave's sums
        tab[(i / G4) * kTabRow + col] = (DYNAMIC ? wave_scale[(col % H) >> 4] : kSH * kSWDefault) * (Wx[i] + bg[col]);
      }
      __syncthreads();

      const int n_steps = phase == 0 ? Lq : La;
#pragma unroll
      for (int ch = 0; ch < 2; ++ch) {
        if (ch >= n_chunks) break;
        const unsigned char* tq = tokq + ch * kChunk * kMaxLq;
        const unsigned char* ta = toka + ch * kChunk * kMaxLa;
#pragma unroll 1
        for (int t = 0; t < n_steps; ++t) {
          int& cur = ch == 0 ? cur0 : cur1;
          const unsigned char* hc = hbuf + cur * kBufB;
          unsigned char* hn = hbuf + spare * kBufB;
          if (phase == 0)
            lstm_step<H>(wh, cst[ch], tab, hc, hn, wave, j, q, k_u, [&](int s) { return int(tq[s * kMaxLq + t]); });
          else
            lstm_step<H>(wh, cst[ch], tab, hc, hn, wave, j, q, k_u,
                         [&](int s) { return t == 0 ? V - 1 : int(ta[s * kMaxLa + t - 1]); });
          __syncthreads();  // h' is complete; nobody reads the old h any more
          const int old = cur;
          cur = spare;
          spare = old;

          if (phase == 1 && wave < 4) {
            // ---- logits of answer position t for sample tile `wave`: rows = outputs, columns = samples ----
            const int s = 16 * wave + j;
            const unsigned char* src = hbuf + cur * kBufB + s * kRowB + 16 * q;
            floatx4 lg = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KS; ++kb) {
              const f16x8 b0 = *reinterpret_cast<const f16x8*>(src + 64 * kb);
              const f16x8 b1 = *reinterpret_cast<const f16x8*>(src + kTermB + 64 * kb);
              const f16x8 w0 = wo_s[0][kb][lane], w1 = wo_s[1][kb][lane];
              lg = __builtin_amdgcn_mfma_f32_16x16x32_f16(w0, b1, lg, 0, 0, 0);
              lg = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1, b0, lg, 0, 0, 0);
              lg = __builtin_amdgcn_mfma_f32_16x16x32_f16(w0, b0, lg, 0, 0, 0);
            }
            float z[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) z[i] = fmaf(lg[i], u_o, bo4[i]);
            const int gs = c0 + ch * kChunk + s;  // sample index in the batch
            const bool valid = gs < a.B;
            if (a.logits && valid) {
              float* out = a.logits + ((static_cast<size_t>(member) * a.B + gs) * La + t) * n_out;
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (4 * q + i < n_out) out[4 * q + i] = z[i];
            }
            // cross-entropy of the true digit: softmax over the rows, i.e. over i and the four q groups
            const int y = ta[s * kMaxLa + t];
            float mx = -INFINITY, picked = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if (4 * q + i < n_out) mx = fmaxf(mx, z[i]);
              if (4 * q + i == y) picked = z[i];
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            float se = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (4 * q + i < n_out) se += __builtin_amdgcn_exp2f(kLog2e * (z[i] - mx));  // one ulp; the terms are at most one
            se += __shfl_xor(se, 16, 64);
            se += __shfl_xor(se, 32, 64);
            picked += __shfl_xor(picked, 16, 64);
            picked += __shfl_xor(picked, 32, 64);
            if (valid && q == 0) loss_acc += (mx + 0.6931471805599453f * __builtin_amdgcn_logf(se)) - picked;  // se in [1, 16]
          }
        }
      }
    }
  }

  // ---- first build: a weight beyond the default scale's range anywhere in the workgroup marks the member ----
  __syncthreads();
  if (!DYNAMIC) {
    if (tid == 0) refetch = 0;
    __syncthreads();
    if (range_max > kSplitMax) refetch = 1;
  }
  // ---- fitness: lanes in a fixed order, then waves 0..3 in order ----
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) loss_acc += __shfl_xor(loss_acc, o, 64);
  if (lane == 0) wave_loss[wave] = loss_acc;
  __syncthreads();
  if (tid == 0) {
    const float total = ((wave_loss[0] + wave_loss[1]) + wave_loss[2]) + wave_loss[3];
    if (a.fitness) a.fitness[member] = -total / (static_cast<float>(a.B) * static_cast<float>(La));
    if (!DYNAMIC && refetch) *mark = __uint_as_float(kMarkBits);
  }
}

int lstm_supported(int V, int H, int n_out, int Lq, int La) {
  EVO_REQUIRE(H == 64 || H == 128, EVO_ERR_UNSUPPORTED, "lstm: hidden width must be 64 or 128 (got %d)", H);
  EVO_REQUIRE(V >= 1 && V <= kMaxV, EVO_ERR_UNSUPPORTED, "lstm: vocabulary must be in [1, %d] (got %d)", kMaxV, V);
  EVO_REQUIRE(n_out >= 1 && n_out <= kMaxOut && n_out <= V, EVO_ERR_UNSUPPORTED,
              "lstm: outputs must be in [1, %d] and, being fed back as tokens, at most V (got %d)", kMaxOut, n_out);
  EVO_REQUIRE(Lq >= 1 && Lq <= kMaxLq && La >= 1 && La <= kMaxLa, EVO_ERR_UNSUPPORTED,
              "lstm: query length must be in [1, %d] and answer length in [1, %d] (got %d, %d)", kMaxLq, kMaxLa, Lq,
              La);
  return EVO_OK;
}

int64_t lstm_param_count(int V, int H, int n_out) {
  return 2 * (static_cast<int64_t>(V) * 4 * H + static_cast<int64_t>(H) * 4 * H + 4 * H) +
         static_cast<int64_t>(H) * n_out + n_out;
}

int launch_lstm_seq2seq(int V, int H, int n_out, const float* params, const int32_t* query, const int32_t* answer,
                        int pop, int B, int Lq, int La, float* fitness, float* logits, hipStream_t s) {
  LstmArgs a;
  a.params = params, a.query = query, a.answer = answer, a.fitness = fitness, a.logits = logits;
  a.P = static_cast<int>(lstm_param_count(V, H, n_out));
  a.B = B, a.Lq = Lq, a.La = La, a.V = V, a.n_out = n_out;
  if (H == 128) {
    hipLaunchKernelGGL((lstm_seq2seq_kernel<128, false>), dim3(pop), dim3(512), 0, s, a);
    hipLaunchKernelGGL((lstm_seq2seq_kernel<128, true>), dim3(pop), dim3(512), 0, s, a);
  } else {
    hipLaunchKernelGGL((lstm_seq2seq_kernel<64, false>), dim3(pop), dim3(256), 0, s, a);
    hipLaunchKernelGGL((lstm_seq2seq_kernel<64, true>), dim3(pop), dim3(256), 0, s, a);
  }
  return check_launch("lstm_seq2seq_kernel");
}

}  // namespace evo
