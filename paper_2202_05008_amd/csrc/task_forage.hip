// The shared-world task: the whole population lives as agents of one world (Section 3, WaterWorld
// paragraph: every member is spawned in the same task roll-out and measured there).  The paper
// gives the scheme, not the rules; the world is this library's own definition, stated in
// include/evo.h (unit square, food and poison items that reappear elsewhere once eaten, sensing of
// the nearest food, poison and other agent, point-mass motion with drag and walls).
//
// Agents of one world see each other's positions of the current step, so a step is a grid-wide
// dependency: one kernel launch per step, positions double-buffered in the task's workspace.
// A launch is a few microseconds of work spread as widely as its parallelism allows:
//   workgroup = 8 agents x 4 worlds, two waves per world (main and helper; the four main waves read
//   the same policy weights);
//   eight lanes per agent: they split the nearest-neighbour scans (each judges two candidates per
//   16-byte LDS read, then a three-stage reduction on (distance, index) by lane moves) and the hidden
//   units of the policy (each an eighth of a layer; the layer's activations go round by lane shuffles);
//   the helper wave stages half of the positions, places the items and keeps their book, scans the item
//   lists and the upper half of the agents, leaves its results in LDS and exits; the main wave scans the
//   lower half, merges, runs the policy, moves its agents and tests the touches.
// Everything that decides an integer -- who is nearest, who touches an item -- is computed in
// binary32 with each operation rounded on its own (no fused multiply-add), as the task defines it.
#include <algorithm>

#include "kernels.h"

#include <atomic>
#include "philox.h"

namespace evo {

constexpr uint32_t kTagAgent = EVO_TAG_WORLD_AGENT;  // Philox streams of the start positions and of the items
constexpr uint32_t kTagItem = EVO_TAG_WORLD_ITEM;
constexpr int kObs = 8;
constexpr int kLanesPerAgent = 8;
constexpr int kAgentsPerBlock = 64 / kLanesPerAgent;  // a wave; the workgroup's waves are worlds
constexpr int kWorldsPerBlock = 4;
constexpr int kStepThreads = 2 * 64 * kWorldsPerBlock;  // per world a main wave and a helper wave

__host__ __device__ constexpr int pad_to(int n, int m) { return (n + m - 1) / m * m; }

struct WorldConst {
  float dt, thrust, drag, vmax, r2;
  int n_food, n_items;
};

struct StepArgs {
  const float* params;  // [pop][P]; unused when actions_in is set
  int P, pop, worlds;
  int act[3];
  WorldConst c;
  uint32_t key0, key1, gen;
  const uint32_t* gen_dev;
  const float2* pos_in;      // [worlds][pop]
  float2* pos_out;           // [worlds][pop]
  const float2* vel_in;      // [worlds][pop]
  float2* vel_out;           // [worlds][pop] (may alias vel_in: an agent's velocity is its own)
  int32_t* reward;           // [worlds][pop]: += this step's reward (accumulate) or = (otherwise)
  int accumulate;
  const uint32_t* counts_in;   // [worlds][n_items]: times each item was eaten before the previous step
  const uint32_t* hits_prev;   // [worlds][n_items] or null: eaten in the previous step
  uint32_t* counts_out;        // [worlds][n_items] or null: counts_in + hits_prev, for the next step
  uint32_t* hits_cur;          // [worlds][n_items]: set to 1 for every item touched in this step (zero on entry)
  uint32_t* hits_clear;        // [worlds][n_items] or null: zeroed for the step after the next
  const float2* actions_in;    // test hook: [worlds][pop] actions instead of the policy's
  float* obs_out;              // test hook: [worlds][pop][8]
};

// Value of the partner lane in the butterfly stages that cover an agent's eight (or sixteen) lanes, as
// data-parallel-primitive moves (register to register, no trip through LDS): stage 0 swaps
// neighbours, stage 1 swaps pairs (both quad permutations), stage 2 mirrors the eight lanes, which
// pairs each lane of one quad with a lane of the other, stage 3 mirrors a row of sixteen lanes.
template <int STAGE>
__device__ __forceinline__ int partner_bits(int x) {
  // quad_perm 1,0,3,2 / quad_perm 2,3,0,1 / row_half_mirror / row_mirror
  constexpr int ctrl = STAGE == 0 ? 0xB1 : STAGE == 1 ? 0x4E : STAGE == 2 ? 0x141 : 0x140;
  // every lane has a partner in these patterns, so the value for lanes without one is never used
  return __builtin_amdgcn_update_dpp(0, x, ctrl, 0xF, 0xF, true);
}
template <int STAGE>
__device__ __forceinline__ float partner(float x) {
  return __int_as_float(partner_bits<STAGE>(__float_as_int(x)));
}
// Value of the lane N places away in the rotation of a row of sixteen lanes (the lanes of one agent when it has
// sixteen), again register to register.  Which way the hardware rotates does not matter to the callers: they
// apply the same move to the lane number to learn whose value they receive.
template <int N>
__device__ __forceinline__ int rotated_bits(int x) {
  static_assert(N >= 1 && N <= 15, "a rotation inside a row");
  return __builtin_amdgcn_update_dpp(0, x, 0x120 + N, 0xF, 0xF, true);  // row_ror:N
}
template <int N>
__device__ __forceinline__ float rotated(float x) {
  return __int_as_float(rotated_bits<N>(__float_as_int(x)));
}

// Sum over an agent's LPA lanes (8 or 16), left in every one of them.
template <int LPA = kLanesPerAgent>
__device__ __forceinline__ float agent_sum(float x) {
  static_assert(LPA == 8 || LPA == 16, "the butterfly covers eight or sixteen lanes");
  x += partner<0>(x);
  x += partner<1>(x);
  x += partner<2>(x);
  if (LPA == 16) x += partner<3>(x);
  return x;
}
template <int LPA = kLanesPerAgent>
__device__ __forceinline__ int agent_sum(int x) {
  x += partner_bits<0>(x);
  x += partner_bits<1>(x);
  x += partner_bits<2>(x);
  if (LPA == 16) x += partner_bits<3>(x);
  return x;
}

// The task's distance: products and sum rounded one by one.
__device__ __forceinline__ float dist2(float dx, float dy) {
#pragma clang fp contract(off)
  const float xx = dx * dx;
  const float yy = dy * dy;
  return xx + yy;
}

// Nearest candidate so far: distance and index (the offset is read back from the index at the end).
struct Nearest {
  float d2;
  int idx;
};

// Candidates arrive in increasing index within a lane: strict "<" keeps the lowest index.
template <bool CHECK>
__device__ __forceinline__ void nearest_offer(Nearest& n, float2 p, float ox, float oy, int idx, int self) {
  const float d2 = dist2(ox - p.x, oy - p.y);
  bool take = d2 < n.d2;
  if (CHECK) take = take && idx != self;
  n.d2 = take ? d2 : n.d2;
  n.idx = take ? idx : n.idx;
}

// 64 candidates: four chunks of 2 per lane and 8 lanes.
__device__ __forceinline__ void load_scan64(float4 (&c)[4], const float2* s, int base, int q) {
#pragma unroll
  for (int k = 0; k < 4; ++k) c[k] = *reinterpret_cast<const float4*>(s + base + k * 2 * kLanesPerAgent + 2 * q);
}

template <bool CHECK>
__device__ __forceinline__ void nearest_scan64(Nearest& n, float2 p, const float4 (&c)[4], int base, int q, int self) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = base + k * 2 * kLanesPerAgent + 2 * q;
    nearest_offer<CHECK>(n, p, c[k].x, c[k].y, i, self);
    nearest_offer<CHECK>(n, p, c[k].z, c[k].w, i + 1, self);
  }
}

// One chunk of candidates, two per lane of the agent (the item lists are short).
__device__ __forceinline__ void nearest_scan16(Nearest& n, float2 p, const float2* s, int base, int q) {
  const float4 c = *reinterpret_cast<const float4*>(s + base + 2 * q);
  nearest_offer<false>(n, p, c.x, c.y, base + 2 * q, -1);
  nearest_offer<false>(n, p, c.z, c.w, base + 2 * q + 1, -1);
}

// Merge over the lanes of an agent (smaller distance, then lower index) and read the offset back.
template <int LPA = kLanesPerAgent>
__device__ __forceinline__ float2 nearest_finish(Nearest n, float2 p, const float2* s, int limit) {
  // smaller distance, then lower index = smaller 64-bit key (distance bits, index): a distance is a sum of
  // squares or the initial infinity, and non-negative floats order like their bit patterns
  auto merge = [&](float od, int oi) {
    const uint64_t mine = (static_cast<uint64_t>(__float_as_uint(n.d2)) << 32) | static_cast<uint32_t>(n.idx);
    const uint64_t other = (static_cast<uint64_t>(__float_as_uint(od)) << 32) | static_cast<uint32_t>(oi);
    const bool take = other < mine;
    n.d2 = take ? od : n.d2;
    n.idx = take ? oi : n.idx;
  };
  merge(partner<0>(n.d2), partner_bits<0>(n.idx));
  merge(partner<1>(n.d2), partner_bits<1>(n.idx));
  merge(partner<2>(n.d2), partner_bits<2>(n.idx));
  if (LPA == 16) merge(partner<3>(n.d2), partner_bits<3>(n.idx));
  if (n.idx >= limit) return make_float2(0.f, 0.f);  // nothing comparable (non-finite positions)
  const float2 o = s[n.idx];
  return make_float2(o.x - p.x, o.y - p.y);
}

__device__ __forceinline__ float tanh_hw(float x) {
  const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);  // e^{2x}
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}

__device__ __forceinline__ float activate(float x, int act) {
  if (act == EVO_ACT_TANH) return tanh_hw(x);
  if (act == EVO_ACT_RELU) return fmaxf(x, 0.f);
  return x;
}

// A lane's slice of the policy's weights (columns c0 .. c0 + HQ - 1 of every layer, rows c0 .. of the
// last one), loaded at the start of the kernel so that the round trip to L2 runs under the scans.
template <int H, int LPA = kLanesPerAgent>
struct PolicySlice {
  static constexpr int HQ = H / LPA;
  static_assert(HQ >= 2 && HQ % 2 == 0, "a lane's columns are loaded two at a time");
  static constexpr int kRows2 = H <= 32 ? H : 8;   // rows of W2 held here; the rest is read when it is used
  // With sixteen lanes per agent and the whole of W2 held here, the rows sit in the order in which the hidden
  // activations reach the lane by rotations of its row: w2[n HQ + v] is the row of activation v of the lane whose
  // value rotation n delivers (n = 0: the lane's own), so layer 2 needs no gather at all.
  static constexpr bool kRotated = LPA == 16 && kRows2 == H;
  float w1[kObs][HQ], b1[HQ], w2[kRows2][HQ], b2[HQ], w3[HQ][2], b3[2];
  const float* rest;  // &W2[kRows2][c0]
};

// Rows of W2 in rotation order (see PolicySlice): rotation N delivers the value of lane `from`.
template <int H, int LPA, int N>
__device__ __forceinline__ void rotated_rows(const float* __restrict__ W2, int q, int c0, PolicySlice<H, LPA>& s) {
  constexpr int HQ = PolicySlice<H, LPA>::HQ;
  if constexpr (N < 16) {
    int from = q;
    if constexpr (N > 0) from = rotated_bits<N>(q);
#pragma unroll
    for (int v = 0; v < HQ; ++v)
#pragma unroll
      for (int u = 0; u < HQ; u += 2) {
        const float2 w = *reinterpret_cast<const float2*>(W2 + (from * HQ + v) * H + c0 + u);
        s.w2[N * HQ + v][u] = w.x, s.w2[N * HQ + v][u + 1] = w.y;
      }
    rotated_rows<H, LPA, N + 1>(W2, q, c0, s);
  }
}
// Layer 2 on activations that arrive by rotation: part[u] += h[from][v] W2[from HQ + v][c0 + u] for every lane of
// the agent in turn.
template <int H, int LPA, int N>
__device__ __forceinline__ void rotated_layer(const PolicySlice<H, LPA>& s, const float (&mine)[H / LPA],
                                              float (&part)[H / LPA]) {
  constexpr int HQ = H / LPA;
  if constexpr (N < 16) {
#pragma unroll
    for (int v = 0; v < HQ; ++v) {
#pragma unroll
      for (int u = 0; u < HQ; ++u) {
        if constexpr (N == 0) {
          part[u] = fmaf(mine[v], s.w2[v][u], part[u]);
        } else {
          // the rotation rides in the multiply-add itself (the compiler keeps it as a move of its own).  A lane
          // move may not read a register in the two instructions after it is written: the first of these
          // statements brings its own wait, the others read registers written long before
          if constexpr (N == 1)
            asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_ror:%3 row_mask:0xf bank_mask:0xf bound_ctrl:0"
                : "+v"(part[u])
                : "v"(mine[v]), "v"(s.w2[N * HQ + v][u]), "n"(N));
          else
            asm("v_fmac_f32_dpp %0, %1, %2 row_ror:%3 row_mask:0xf bank_mask:0xf bound_ctrl:0"
                : "+v"(part[u])
                : "v"(mine[v]), "v"(s.w2[N * HQ + v][u]), "n"(N));
        }
      }
    }
    rotated_layer<H, LPA, N + 1>(s, mine, part);
  }
}

template <int H, int LPA>
__device__ __forceinline__ void policy_load(const float* __restrict__ th, int q, PolicySlice<H, LPA>& s) {
  constexpr int HQ = PolicySlice<H, LPA>::HQ;
  const int c0 = q * HQ;
  const float* W1 = th;
  const float* b1 = W1 + kObs * H;
  const float* W2 = b1 + H;
  const float* b2 = W2 + H * H;
  const float* W3 = b2 + H;
  const float* b3 = W3 + H * 2;
  auto row = [&](const float* src, float (&dst)[HQ]) {
#pragma unroll
    for (int u = 0; u < HQ; u += 2) {
      const float2 w = *reinterpret_cast<const float2*>(src + c0 + u);
      dst[u] = w.x, dst[u + 1] = w.y;
    }
  };
#pragma unroll
  for (int i = 0; i < kObs; ++i) row(W1 + i * H, s.w1[i]);
  row(b1, s.b1);
  if constexpr (PolicySlice<H, LPA>::kRotated) {
    rotated_rows<H, LPA, 0>(W2, q, c0, s);
  } else {
#pragma unroll
    for (int i = 0; i < PolicySlice<H, LPA>::kRows2; ++i) row(W2 + i * H, s.w2[i]);
  }
  s.rest = W2 + PolicySlice<H, LPA>::kRows2 * H + c0;
  row(b2, s.b2);
#pragma unroll
  for (int u = 0; u < HQ; ++u) {
    const float2 w = *reinterpret_cast<const float2*>(W3 + (c0 + u) * 2);
    s.w3[u][0] = w.x, s.w3[u][1] = w.y;
  }
  s.b3[0] = b3[0], s.b3[1] = b3[1];
}

// All H activations of a layer to every lane of the agent.
template <int H, int LPA>
__device__ __forceinline__ void gather_agent(const float (&mine)[H / LPA], int lane, float (&full)[H]) {
  constexpr int HQ = H / LPA;
#pragma unroll
  for (int s = 0; s < LPA; ++s)
#pragma unroll
    for (int u = 0; u < HQ; ++u) full[s * HQ + u] = __shfl(mine[u], (lane & ~(LPA - 1)) | s);
}

// The policy of dims (8, H, H, 2) for one agent; every lane of the agent returns both outputs.
// TANH: all three activations are tanh (the usual policy), known when the kernel is built: no switch per value.
template <int H, int LPA, bool TANH = false>
__device__ __forceinline__ float2 policy_forward(const PolicySlice<H, LPA>& s, const int (&act_rt)[3], int lane,
                                                 const float (&obs)[kObs]) {
  const int act[3] = {TANH ? EVO_ACT_TANH : act_rt[0], TANH ? EVO_ACT_TANH : act_rt[1],
                      TANH ? EVO_ACT_TANH : act_rt[2]};
  constexpr int HQ = PolicySlice<H, LPA>::HQ;
  float part[HQ], full[H];
#pragma unroll
  for (int u = 0; u < HQ; ++u) part[u] = s.b1[u];
#pragma unroll
  for (int i = 0; i < kObs; ++i)
#pragma unroll
    for (int u = 0; u < HQ; ++u) part[u] = fmaf(obs[i], s.w1[i][u], part[u]);
#pragma unroll
  for (int u = 0; u < HQ; ++u) part[u] = activate(part[u], act[0]);
  if constexpr (PolicySlice<H, LPA>::kRotated) {
    float h1[HQ];
#pragma unroll
    for (int u = 0; u < HQ; ++u) h1[u] = part[u], part[u] = s.b2[u];
    rotated_layer<H, LPA, 0>(s, h1, part);
  } else {
    gather_agent<H, LPA>(part, lane, full);
#pragma unroll
    for (int u = 0; u < HQ; ++u) part[u] = s.b2[u];
#pragma unroll
    for (int i = 0; i < PolicySlice<H, LPA>::kRows2; ++i)
#pragma unroll
      for (int u = 0; u < HQ; ++u) part[u] = fmaf(full[i], s.w2[i][u], part[u]);
#pragma unroll 16
    for (int i = PolicySlice<H, LPA>::kRows2; i < H; ++i)
#pragma unroll
      for (int u = 0; u < HQ; u += 2) {
        const float2 w = *reinterpret_cast<const float2*>(s.rest + (i - PolicySlice<H, LPA>::kRows2) * H + u);
        part[u] = fmaf(full[i], w.x, part[u]);
        part[u + 1] = fmaf(full[i], w.y, part[u + 1]);
      }
  }
#pragma unroll
  for (int u = 0; u < HQ; ++u) part[u] = activate(part[u], act[1]);
  float o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int u = 0; u < HQ; ++u) {
    o0 = fmaf(part[u], s.w3[u][0], o0);
    o1 = fmaf(part[u], s.w3[u][1], o1);
  }
  o0 = agent_sum<LPA>(o0), o1 = agent_sum<LPA>(o1);
  return make_float2(activate(o0 + s.b3[0], act[2]), activate(o1 + s.b3[1], act[2]));
}

// One axis of the motion: new velocity and position, each operation rounded on its own.
__device__ __forceinline__ void move_axis(const WorldConst& c, float a, float& p, float& v) {
#pragma clang fp contract(off)
  a = fminf(fmaxf(a, -1.f), 1.f);
  const float dv = c.drag * v;
  const float da = c.thrust * a;
  float nv = dv + da;
  nv = fminf(fmaxf(nv, -c.vmax), c.vmax);
  const float step = c.dt * nv;
  float np = p + step;
  if (np < 0.f) np = 0.f, nv = 0.f;
  if (np > 1.f) np = 1.f, nv = 0.f;
  p = np, v = nv;
}

// Touches of one list of items (16 slots per chunk); returns how many this lane found.
__device__ __forceinline__ int touch_scan(const WorldConst& c, float2 p, const float2* s, int padded, int q,
                                          uint32_t* hits) {
  int found = 0;
  for (int base = 0; base < padded; base += 2 * kLanesPerAgent) {
    const float4 it = *reinterpret_cast<const float4*>(s + base + 2 * q);
    if (dist2(it.x - p.x, it.y - p.y) <= c.r2) ++found, atomicOr(hits + base + 2 * q, 1u);
    if (dist2(it.z - p.x, it.w - p.y) <= c.r2) ++found, atomicOr(hits + base + 2 * q + 1, 1u);
  }
  return found;
}

// Per lane of a helper wave, for the main wave of the same world: its part of the agent scan and the
// two item offsets, as six words (structure of arrays: word w of lane l at [w][l]).
constexpr int kExchangeWords = 6;

template <int H, bool TANH>
__global__ __launch_bounds__(kStepThreads) void world_step_kernel(StepArgs a) {
  extern __shared__ float4 lds4[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int slot = wave & (kWorldsPerBlock - 1);  // which of the workgroup's worlds
  const bool helper = wave >= kWorldsPerBlock;    // waves 4..7 assist waves 0..3
  const int q = lane & (kLanesPerAgent - 1);
  const int agent0 = blockIdx.x * kAgentsPerBlock;
  const int agent = agent0 + lane / kLanesPerAgent;
  const int world = blockIdx.y * kWorldsPerBlock + slot;
  const bool world_live = world < a.worlds;
  const bool live = world_live && agent < a.pop;
  const int n_food = a.c.n_food, n_items = a.c.n_items;
  const int pop_pad = pad_to(a.pop, 64), food_pad = pad_to(n_food, 16), poison_pad = pad_to(n_items - n_food, 16);
  const int region = pop_pad + food_pad + poison_pad;
  // a world's region: every agent, the food, the poison; unused slots lie infinitely far away
  float2* s_pos = reinterpret_cast<float2*>(lds4) + slot * region;
  float2* s_food = s_pos + pop_pad;
  float2* s_poison = s_food + food_pad;
  float* s_xch = reinterpret_cast<float*>(reinterpret_cast<float2*>(lds4) + kWorldsPerBlock * region) +
                 slot * kExchangeWords * 64;
  if (a.gen_dev) a.gen = *a.gen_dev;
  const float inf = __builtin_inff();

  PolicySlice<H> weights;
  if (world_live) {
    const float2* pin = a.pos_in + static_cast<size_t>(world) * a.pop;
    const int role = helper ? 1 : 0;
    float2 t[8];  // the two waves of a world stage alternate runs of 64 positions: eight loads in flight each
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = (2 * k + role) * 64 + lane;
      t[k] = pin[min(j, a.pop - 1)];  // in bounds; slots past the last agent are replaced when they are stored
    }
    // main wave: the policy's weights, requested behind the positions; their round trip to L2 runs under
    // everything up to the forward pass
    if (!helper && live && !a.actions_in) policy_load<H>(a.params + static_cast<size_t>(agent) * a.P, q, weights);
    if (helper) {  // the items and their book
      for (int sl = lane; sl < food_pad + poison_pad; sl += 64) {
        const bool is_food = sl < food_pad;
        const int i = is_food ? sl : n_food + sl - food_pad;
        float2 where = make_float2(inf, inf);
        if (i < (is_food ? n_food : n_items)) {
          const size_t o = static_cast<size_t>(world) * n_items + i;
          uint32_t cnt = a.counts_in[o];
          if (a.hits_prev) cnt += a.hits_prev[o];
          if (blockIdx.x == 0) {  // one workgroup per world keeps the item book
            if (a.counts_out) a.counts_out[o] = cnt;
            if (a.hits_clear) a.hits_clear[o] = 0u;
          }
          const u32x4 w = philox4x32_10(256u * cnt + static_cast<uint32_t>(i), static_cast<uint32_t>(world), a.gen,
                                        kTagItem, a.key0, a.key1);
          where = make_float2(unit_open(w.x), unit_open(w.y));
        }
        s_food[sl] = where;  // the poison list follows the food list
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = (2 * k + role) * 64 + lane;
      if (j < pop_pad) s_pos[j] = j < a.pop ? t[k] : make_float2(inf, inf);  // the first use of the loaded values
    }
    for (int j = 1024 + role * 64 + lane; j < pop_pad; j += 128) s_pos[j] = j < a.pop ? pin[j] : make_float2(inf, inf);
  }
  __syncthreads();

  // The agent scan is shared: the main wave takes the first blocks of 64 candidates, the helper the rest
  // and the two item lists (about two blocks' worth of work).
  const int blocks = pop_pad / 64;
  const int main_blocks = min(blocks, (blocks + 3) / 2);
  const size_t me = static_cast<size_t>(world) * a.pop + min(agent, a.pop - 1);
  float2 p = make_float2(0.f, 0.f), v = p;
  Nearest other{inf, 0x7fffffff};
  float2 f = p, g = p;
  if (live) {
    p = s_pos[agent];
    const int own_block = agent0 & ~63;  // the only 64 candidates that hold agents of this wave
    // two sets of 64 candidates take turns: one is on its way from LDS while the other is judged
    auto judge = [&](const float4 (&c)[4], int base) {
      if (base == own_block)
        nearest_scan64<true>(other, p, c, base, q, agent);
      else
        nearest_scan64<false>(other, p, c, base, q, agent);
    };
    const int first = helper ? main_blocks * 64 : 0, last = helper ? pop_pad : main_blocks * 64;
    float4 ping[4], pong[4];
    if (first < last) load_scan64(ping, s_pos, first, q);
    for (int base = first; base < last; base += 128) {
      const bool second = base + 64 < last;
      if (second) load_scan64(pong, s_pos, base + 64, q);
      judge(ping, base);
      if (base + 128 < last) load_scan64(ping, s_pos, base + 128, q);
      if (second) judge(pong, base + 64);
    }
    if (helper) {
      Nearest food{inf, 0x7fffffff}, poison{inf, 0x7fffffff};
      for (int base = 0; base < food_pad; base += 16) nearest_scan16(food, p, s_food, base, q);
      for (int base = 0; base < poison_pad; base += 16) nearest_scan16(poison, p, s_poison, base, q);
      f = nearest_finish(food, p, s_food, food_pad);
      g = nearest_finish(poison, p, s_poison, poison_pad);
      s_xch[0 * 64 + lane] = other.d2;
      s_xch[1 * 64 + lane] = __int_as_float(other.idx);
      s_xch[2 * 64 + lane] = f.x, s_xch[3 * 64 + lane] = f.y;
      s_xch[4 * 64 + lane] = g.x, s_xch[5 * 64 + lane] = g.y;
    } else {
      v = a.vel_in[me];
    }
  }
  __syncthreads();
  if (helper || !live) return;  // no barrier below this line

  {  // the helper's candidates all have higher indices: they win only when strictly nearer
    const float hd = s_xch[0 * 64 + lane];
    const int hi = __float_as_int(s_xch[1 * 64 + lane]);
    const bool take = hd < other.d2;
    other.d2 = take ? hd : other.d2;
    other.idx = take ? hi : other.idx;
    f = make_float2(s_xch[2 * 64 + lane], s_xch[3 * 64 + lane]);
    g = make_float2(s_xch[4 * 64 + lane], s_xch[5 * 64 + lane]);
  }
  const float2 o = nearest_finish(other, p, s_pos, pop_pad);

  const float obs[kObs] = {v.x, v.y, f.x, f.y, g.x, g.y, o.x, o.y};
  if (a.obs_out && q == 0) {
    float4* dst = reinterpret_cast<float4*>(a.obs_out + me * kObs);
    dst[0] = make_float4(obs[0], obs[1], obs[2], obs[3]);
    dst[1] = make_float4(obs[4], obs[5], obs[6], obs[7]);
  }
  float2 action;
  if (a.actions_in)
    action = a.actions_in[me];
  else
    action = policy_forward<H, kLanesPerAgent, TANH>(weights, a.act, lane, obs);

  move_axis(a.c, action.x, p.x, v.x);
  move_axis(a.c, action.y, p.y, v.y);

  uint32_t* hits = a.hits_cur + static_cast<size_t>(world) * n_items;
  int reward = touch_scan(a.c, p, s_food, food_pad, q, hits) - touch_scan(a.c, p, s_poison, poison_pad, q, hits + n_food);
  reward = agent_sum(reward);
  if (q == 0) {
    a.pos_out[me] = p;
    a.vel_out[me] = v;
    a.reward[me] = a.accumulate ? a.reward[me] + reward : reward;
  }
}

// ---- single-agent form: every member alone in its own copy of each world ---------------------------------
// Nothing couples the members, so the whole episode runs in one launch (the fused roll-out of the control
// tasks): wave = 64 / LPA members x LPA lanes in one world (sixteen lanes where the hidden width allows it:
// twice the waves and half the length of a member's dependent chain), the policy's weights in registers for
// all steps, each member's item lists and item book in LDS.  A touched item is moved at once by the lane
// that found it (every slot is judged by exactly one lane per step, after the step's sensing), which is
// "from the next step on".  All members start at agent 0's place among the same items.
struct SoloArgs {
  const float* params;  // [pop][P]
  int P, pop, worlds, steps;
  int act[3];
  WorldConst c;
  uint32_t key0, key1, gen;
  const uint32_t* gen_dev;
  int32_t* reward;       // [worlds][pop]: the episode's summed reward
  float2* pos_out;       // [worlds][pop] or null: state after the last step
  float2* vel_out;       // [worlds][pop] or null
  uint32_t* counts_out;  // [worlds][pop][n_items] or null: times each item was eaten
};

template <int H, int LPA, bool TANH>
__global__ __launch_bounds__(64 * kWorldsPerBlock) void world_solo_kernel(SoloArgs a) {
  constexpr int kMembers = 64 / LPA;  // members per wave
  extern __shared__ float4 lds4[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int q = lane & (LPA - 1), la = lane / LPA;
  const int agent = blockIdx.x * kMembers + la;
  const int world = blockIdx.y * kWorldsPerBlock + wave;
  const bool live = world < a.worlds && agent < a.pop;
  const int n_food = a.c.n_food, n_items = a.c.n_items;
  const int food_pad = pad_to(n_food, 2 * LPA), poison_pad = pad_to(n_items - n_food, 2 * LPA);
  const int slots = food_pad + poison_pad;
  // per wave: [members][slots] positions, then [members][slots] counts
  float2* s_item = reinterpret_cast<float2*>(lds4) + wave * kMembers * slots;
  uint32_t* s_count = reinterpret_cast<uint32_t*>(reinterpret_cast<float2*>(lds4) + kWorldsPerBlock * kMembers * slots) +
                      wave * kMembers * slots;
  if (a.gen_dev) a.gen = *a.gen_dev;
  const float inf = __builtin_inff();
  auto item_of = [&](int slot) {  // item index of a slot of the two padded lists, or -1
    const bool is_food = slot < food_pad;
    const int i = is_food ? slot : n_food + slot - food_pad;
    return i < (is_food ? n_food : n_items) ? i : -1;
  };
  auto place = [&](int i, uint32_t cnt) {
    const u32x4 w = philox4x32_10(256u * cnt + static_cast<uint32_t>(i), static_cast<uint32_t>(world), a.gen, kTagItem,
                                  a.key0, a.key1);
    return make_float2(unit_open(w.x), unit_open(w.y));
  };

  PolicySlice<H, LPA> weights;
  if (live) policy_load<H, LPA>(a.params + static_cast<size_t>(agent) * a.P, q, weights);
  if (world < a.worlds) {  // the same fresh items for every member of the wave
    for (int slot = lane; slot < slots; slot += 64) {
      const int i = item_of(slot);
      const float2 where = i >= 0 ? place(i, 0u) : make_float2(inf, inf);
      for (int m = 0; m < kMembers; ++m) s_item[m * slots + slot] = where, s_count[m * slots + slot] = 0u;
    }
  }
  __syncthreads();
  if (!live) return;  // no barrier below this line; the lanes of a member stay together

  float2* my_food = s_item + la * slots;
  float2* my_poison = my_food + food_pad;
  uint32_t* my_count = s_count + la * slots;
  float2 p, v = make_float2(0.f, 0.f);
  {
    const u32x4 w = philox4x32_10(0u, static_cast<uint32_t>(world), a.gen, kTagAgent, a.key0, a.key1);
    p = make_float2(unit_open(w.x), unit_open(w.y));
  }
  int reward = 0;
#pragma unroll 1
  for (int step = 0; step < a.steps; ++step) {
    Nearest food{inf, 0x7fffffff}, poison{inf, 0x7fffffff};
    for (int base = 0; base < food_pad; base += 2 * LPA) nearest_scan16(food, p, my_food, base, q);
    for (int base = 0; base < poison_pad; base += 2 * LPA) nearest_scan16(poison, p, my_poison, base, q);
    const float2 f = nearest_finish<LPA>(food, p, my_food, food_pad);
    const float2 g = nearest_finish<LPA>(poison, p, my_poison, poison_pad);
    const float obs[kObs] = {v.x, v.y, f.x, f.y, g.x, g.y, 0.f, 0.f};  // nobody else is there
    const float2 action = policy_forward<H, LPA, TANH>(weights, a.act, lane, obs);
    move_axis(a.c, action.x, p.x, v.x);
    move_axis(a.c, action.y, p.y, v.y);
    // touches: the lane that judges a slot also moves the item it finds eaten
    for (int base = 0; base < slots; base += 2 * LPA) {
      const float4 it = *reinterpret_cast<const float4*>(my_food + base + 2 * q);
      const bool hit0 = dist2(it.x - p.x, it.y - p.y) <= a.c.r2, hit1 = dist2(it.z - p.x, it.w - p.y) <= a.c.r2;
      if (hit0 || hit1) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          if (k == 0 ? hit0 : hit1) {
            const int slot = base + 2 * q + k, i = item_of(slot);
            reward += slot < food_pad ? 1 : -1;
            const uint32_t cnt = my_count[slot] + 1u;
            my_count[slot] = cnt;
            my_food[slot] = place(i, cnt);
          }
        }
      }
    }
    // the next step's sensing reads what this step's touches wrote (same wave: LDS keeps program order)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  reward = agent_sum<LPA>(reward);
  const size_t me = static_cast<size_t>(world) * a.pop + agent;
  if (q == 0) {
    a.reward[me] = reward;
    if (a.pos_out) a.pos_out[me] = p;
    if (a.vel_out) a.vel_out[me] = v;
  }
  if (a.counts_out)
    for (int slot = q; slot < slots; slot += LPA) {
      const int i = item_of(slot);
      if (i >= 0) a.counts_out[me * n_items + i] = my_count[slot];
    }
}

struct ResetArgs {
  int pop, worlds, n_items;
  uint32_t key0, key1, gen;
  const uint32_t* gen_dev;
  float2* pos;       // [worlds][pop]
  float2* vel;       // [worlds][pop]
  int32_t* reward;   // [worlds][pop]
  uint32_t* book;    // counts[2] and hits[3]: 5 x [worlds][n_items], all zero at the start
};

__global__ __launch_bounds__(256) void world_reset_kernel(ResetArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (a.gen_dev) a.gen = *a.gen_dev;
  if (i < a.worlds * a.pop) {
    const uint32_t world = i / a.pop, agent = i % a.pop;
    const u32x4 w = philox4x32_10(agent, world, a.gen, kTagAgent, a.key0, a.key1);
    a.pos[i] = make_float2(unit_open(w.x), unit_open(w.y));
    a.vel[i] = make_float2(0.f, 0.f);
    a.reward[i] = 0;
  }
  if (i < 5 * a.worlds * a.n_items) a.book[i] = 0u;
}

// fitness[a] = mean over the worlds of the summed reward (an exact integer sum, one division).
__global__ __launch_bounds__(256) void world_finish_kernel(const int32_t* reward, int pop, int worlds, float* fitness) {
  const int agent = blockIdx.x * 256 + threadIdx.x;
  if (agent >= pop) return;
  int sum = 0;
  for (int r = 0; r < worlds; ++r) sum += reward[static_cast<size_t>(r) * pop + agent];
  fitness[agent] = static_cast<float>(sum) / static_cast<float>(worlds);
}

__global__ __launch_bounds__(256) void world_fill_kernel(uint32_t* dst, int n, uint32_t value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = value;
}

// counts_out = counts + hits (the book after the last step), for the state hook.
__global__ __launch_bounds__(256) void world_counts_kernel(const uint32_t* counts, const uint32_t* hits, int n,
                                                           uint32_t* out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = counts[i] + hits[i];
}

struct Layout {
  size_t pos[2], vel, reward, book, bytes;  // byte offsets into the workspace
};

static Layout carve(int pop, int worlds, int n_items) {
  const size_t agents = static_cast<size_t>(pop) * worlds;
  auto up = [](size_t n) { return (n + 255) & ~size_t(255); };
  Layout l;
  size_t o = 0;
  l.pos[0] = o, o += up(agents * sizeof(float2));
  l.pos[1] = o, o += up(agents * sizeof(float2));
  l.vel = o, o += up(agents * sizeof(float2));
  l.reward = o, o += up(agents * sizeof(int32_t));
  l.book = o, o += up(5 * static_cast<size_t>(worlds) * n_items * sizeof(uint32_t));
  l.bytes = o;
  return l;
}

constexpr size_t kMaxLdsBytes = 160 * 1024;  // per workgroup on this chip

static size_t step_lds_bytes(int pop, int n_food, int n_items) {
  return static_cast<size_t>(kWorldsPerBlock) *
         ((pad_to(pop, 64) + pad_to(n_food, 16) + pad_to(n_items - n_food, 16)) * sizeof(float2) +
          kExchangeWords * 64 * sizeof(float));
}

static int fill_const(const float* cp, WorldConst* c) {
  c->dt = cp[0], c->thrust = cp[1], c->drag = cp[2], c->vmax = cp[3];
  c->r2 = cp[4] * cp[4];  // the squared touch radius, rounded once
  c->n_food = static_cast<int>(cp[5]);
  c->n_items = c->n_food + static_cast<int>(cp[6]);
  EVO_REQUIRE(cp[5] == static_cast<float>(c->n_food) && cp[6] == static_cast<float>(c->n_items - c->n_food),
              EVO_ERR_ARG, "forage: cp[5] (food items) and cp[6] (poison items) must be whole numbers");
  EVO_REQUIRE(c->n_food >= 1 && c->n_items > c->n_food && c->n_items <= 256, EVO_ERR_ARG,
              "forage: needs at least one food and one poison item and at most 256 items (got %d + %d)", c->n_food,
              c->n_items - c->n_food);
  EVO_REQUIRE(cp[0] > 0.f && cp[1] >= 0.f && cp[2] >= 0.f && cp[2] <= 1.f && cp[3] > 0.f && cp[4] > 0.f, EVO_ERR_ARG,
              "forage: needs dt > 0, thrust >= 0, drag in [0,1], vmax > 0, radius > 0");
  return EVO_OK;
}

template <int H, bool TANH>
static int launch_step_built(const StepArgs& a, hipStream_t s) {
  const dim3 grid((a.pop + kAgentsPerBlock - 1) / kAgentsPerBlock, (a.worlds + kWorldsPerBlock - 1) / kWorldsPerBlock);
  // more than 64 KB of dynamic LDS has to be asked for, once per kernel and device
  static std::atomic<bool> raised[64];  // zero-initialised; a second setter does the same harmless call
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e == hipSuccess && device >= 0 && device < 64 && !raised[device].load()) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&world_step_kernel<H, TANH>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kMaxLdsBytes));
    raised[device].store(e == hipSuccess);
  }
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "forage: raising the LDS limit of the step kernel failed: %s",
              hipGetErrorString(e));
  hipLaunchKernelGGL((world_step_kernel<H, TANH>), grid, dim3(kStepThreads),
                     step_lds_bytes(a.pop, a.c.n_food, a.c.n_items), s, a);
  return check_launch("world_step_kernel");
}
template <int H>
static int launch_step(const StepArgs& a, hipStream_t s) {
  const bool all_tanh = a.act[0] == EVO_ACT_TANH && a.act[1] == EVO_ACT_TANH && a.act[2] == EVO_ACT_TANH;
  return all_tanh ? launch_step_built<H, true>(a, s) : launch_step_built<H, false>(a, s);
}

static int launch_step_for(int H, const StepArgs& a, hipStream_t s) {
  switch (H) {
    case 16: return launch_step<16>(a, s);
    case 32: return launch_step<32>(a, s);
    case 64: return launch_step<64>(a, s);
  }
  return fail(EVO_ERR_UNSUPPORTED, "forage: the hidden width must be 16, 32 or 64");
}

int forage_supported(const MlpShape& sh, int pop, int worlds, const float* cp) {
  WorldConst c;
  int rc = fill_const(cp, &c);
  if (rc) return rc;
  EVO_REQUIRE(sh.n_layers == 3 && sh.dims[0] == kObs && sh.dims[3] == 2 && sh.dims[1] == sh.dims[2] &&
                  (sh.dims[1] == 16 || sh.dims[1] == 32 || sh.dims[1] == 64),
              EVO_ERR_UNSUPPORTED, "forage: the policy must be an MLP of dims {8, H, H, 2} with H = 16, 32 or 64");
  EVO_REQUIRE(pop >= 2, EVO_ERR_ARG, "forage: a world needs at least two agents (got pop = %d)", pop);
  EVO_REQUIRE(worlds >= 1 && worlds <= 4096, EVO_ERR_ARG, "forage: n_rollouts (worlds) must be in [1, 4096]");
  const size_t lds = step_lds_bytes(pop, c.n_food, c.n_items);
  EVO_REQUIRE(lds <= kMaxLdsBytes, EVO_ERR_UNSUPPORTED,
              "forage: too many agents per world: staging the positions of four worlds takes %zu bytes of LDS, %zu fit",
              lds, kMaxLdsBytes);
  return EVO_OK;
}

size_t forage_workspace_bytes(int pop, int worlds, const float* cp) {
  WorldConst c;
  if (fill_const(cp, &c) || pop < 1 || worlds < 1) return 0;
  return carve(pop, worlds, c.n_items).bytes;
}

int launch_forage(const MlpShape& sh, const float* params, int pop, int worlds, int steps, const float* cp,
                  uint64_t seed, uint32_t gen, const uint32_t* gen_dev, void* work, float* fitness, float* pos_out,
                  float* vel_out, int32_t* reward_out, uint32_t* counts_out, hipStream_t s) {
  WorldConst c;
  int rc = fill_const(cp, &c);
  if (rc) return rc;
  const Layout l = carve(pop, worlds, c.n_items);
  char* base = static_cast<char*>(work);
  float2* pos[2] = {reinterpret_cast<float2*>(base + l.pos[0]), reinterpret_cast<float2*>(base + l.pos[1])};
  float2* vel = reinterpret_cast<float2*>(base + l.vel);
  int32_t* reward = reinterpret_cast<int32_t*>(base + l.reward);
  uint32_t* book = reinterpret_cast<uint32_t*>(base + l.book);
  const size_t nb = static_cast<size_t>(worlds) * c.n_items;  // one page of the item book
  uint32_t* counts[2] = {book, book + nb};
  uint32_t* hits[3] = {book + 2 * nb, book + 3 * nb, book + 4 * nb};

  ResetArgs ra;
  ra.pop = pop, ra.worlds = worlds, ra.n_items = c.n_items;
  ra.key0 = static_cast<uint32_t>(seed), ra.key1 = static_cast<uint32_t>(seed >> 32), ra.gen = gen, ra.gen_dev = gen_dev;
  ra.pos = pos[0], ra.vel = vel, ra.reward = reward, ra.book = book;
  const int n_reset = static_cast<int>(std::max(static_cast<size_t>(worlds) * pop, 5 * nb));
  hipLaunchKernelGGL(world_reset_kernel, dim3((n_reset + 255) / 256), dim3(256), 0, s, ra);
  rc = check_launch("world_reset_kernel");
  if (rc) return rc;

  StepArgs a;
  a.params = params, a.P = sh.P, a.pop = pop, a.worlds = worlds;
  a.act[0] = sh.act[0], a.act[1] = sh.act[1], a.act[2] = sh.act[2];
  a.c = c;
  a.key0 = ra.key0, a.key1 = ra.key1, a.gen = gen, a.gen_dev = gen_dev;
  a.vel_in = vel, a.vel_out = vel, a.reward = reward, a.accumulate = 1;
  a.actions_in = nullptr, a.obs_out = nullptr;
  for (int t = 0; t < steps; ++t) {
    a.pos_in = pos[t & 1], a.pos_out = pos[(t + 1) & 1];
    a.counts_in = counts[t & 1], a.counts_out = counts[(t + 1) & 1];
    a.hits_prev = t > 0 ? hits[(t + 2) % 3] : nullptr;  // the page written by step t - 1
    a.hits_cur = hits[t % 3], a.hits_clear = hits[(t + 1) % 3];
    rc = launch_step_for(sh.dims[1], a, s);
    if (rc) return rc;
  }
  if (fitness) {
    hipLaunchKernelGGL(world_finish_kernel, dim3((pop + 255) / 256), dim3(256), 0, s, reward, pop, worlds, fitness);
    rc = check_launch("world_finish_kernel");
    if (rc) return rc;
  }
  // state after the last step, for the test hook
  const size_t agents = static_cast<size_t>(worlds) * pop;
  hipError_t e = hipSuccess;
  if (pos_out) e = hipMemcpyAsync(pos_out, pos[steps & 1], agents * sizeof(float2), hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && vel_out) e = hipMemcpyAsync(vel_out, vel, agents * sizeof(float2), hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && reward_out)
    e = hipMemcpyAsync(reward_out, reward, agents * sizeof(int32_t), hipMemcpyDeviceToDevice, s);
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "forage: copying the final state failed: %s", hipGetErrorString(e));
  if (counts_out) {
    // step steps - 1 read counts[(steps - 1) & 1] + hits of step steps - 2 into counts[steps & 1]; its own hits are
    // in hits[(steps - 1) % 3]
    hipLaunchKernelGGL(world_counts_kernel, dim3((static_cast<int>(nb) + 255) / 256), dim3(256), 0, s,
                       counts[steps & 1], hits[(steps - 1) % 3], static_cast<int>(nb), counts_out);
    rc = check_launch("world_counts_kernel");
    if (rc) return rc;
  }
  return EVO_OK;
}

// Lanes per member of the episode kernel: sixteen where a lane then still owns two columns of a layer.
constexpr int solo_lanes(int H) { return H >= 32 ? 16 : 8; }

static size_t solo_lds_bytes(int n_food, int n_items, int lanes) {
  const size_t slots = pad_to(n_food, 2 * lanes) + pad_to(n_items - n_food, 2 * lanes);
  return static_cast<size_t>(kWorldsPerBlock) * (64 / lanes) * slots * (sizeof(float2) + sizeof(uint32_t));
}

template <int H, bool TANH>
static int launch_solo_built(const SoloArgs& a, hipStream_t s) {
  constexpr int LPA = solo_lanes(H);
  const size_t lds = solo_lds_bytes(a.c.n_food, a.c.n_items, LPA);
  static std::atomic<bool> raised[64];  // zero-initialised; a second setter does the same harmless call
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e == hipSuccess && device >= 0 && device < 64 && !raised[device].load()) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&world_solo_kernel<H, LPA, TANH>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kMaxLdsBytes));
    raised[device].store(e == hipSuccess);
  }
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "forage: raising the LDS limit of the episode kernel failed: %s",
              hipGetErrorString(e));
  constexpr int members = 64 / LPA;
  const dim3 grid((a.pop + members - 1) / members, (a.worlds + kWorldsPerBlock - 1) / kWorldsPerBlock);
  hipLaunchKernelGGL((world_solo_kernel<H, LPA, TANH>), grid, dim3(64 * kWorldsPerBlock), lds, s, a);
  return check_launch("world_solo_kernel");
}
template <int H>
static int launch_solo(const SoloArgs& a, hipStream_t s) {
  const bool all_tanh = a.act[0] == EVO_ACT_TANH && a.act[1] == EVO_ACT_TANH && a.act[2] == EVO_ACT_TANH;
  return all_tanh ? launch_solo_built<H, true>(a, s) : launch_solo_built<H, false>(a, s);
}

int forage_solo_supported(const MlpShape& sh, int pop, int worlds, const float* cp) {
  WorldConst c;
  int rc = fill_const(cp, &c);
  if (rc) return rc;
  EVO_REQUIRE(sh.n_layers == 3 && sh.dims[0] == kObs && sh.dims[3] == 2 && sh.dims[1] == sh.dims[2] &&
                  (sh.dims[1] == 16 || sh.dims[1] == 32 || sh.dims[1] == 64),
              EVO_ERR_UNSUPPORTED, "forage: the policy must be an MLP of dims {8, H, H, 2} with H = 16, 32 or 64");
  EVO_REQUIRE(pop >= 1, EVO_ERR_ARG, "forage: pop must be positive (got %d)", pop);
  EVO_REQUIRE(worlds >= 1 && worlds <= 4096, EVO_ERR_ARG, "forage: n_rollouts (worlds) must be in [1, 4096]");
  EVO_REQUIRE(solo_lds_bytes(c.n_food, c.n_items, solo_lanes(sh.dims[1])) <= kMaxLdsBytes, EVO_ERR_UNSUPPORTED,
              "forage: too many items");
  return EVO_OK;
}

size_t forage_solo_workspace_bytes(int pop, int worlds) {
  if (pop < 1 || worlds < 1) return 0;
  return (static_cast<size_t>(pop) * worlds * sizeof(int32_t) + 255) & ~size_t(255);
}

int launch_forage_solo(const MlpShape& sh, const float* params, int pop, int worlds, int steps, const float* cp,
                       uint64_t seed, uint32_t gen, const uint32_t* gen_dev, void* work, float* fitness, float* pos_out,
                       float* vel_out, int32_t* reward_out, uint32_t* counts_out, hipStream_t s) {
  SoloArgs a;
  int rc = fill_const(cp, &a.c);
  if (rc) return rc;
  a.params = params, a.P = sh.P, a.pop = pop, a.worlds = worlds, a.steps = steps;
  a.act[0] = sh.act[0], a.act[1] = sh.act[1], a.act[2] = sh.act[2];
  a.key0 = static_cast<uint32_t>(seed), a.key1 = static_cast<uint32_t>(seed >> 32), a.gen = gen, a.gen_dev = gen_dev;
  a.reward = static_cast<int32_t*>(work);
  a.pos_out = reinterpret_cast<float2*>(pos_out), a.vel_out = reinterpret_cast<float2*>(vel_out);
  a.counts_out = counts_out;
  switch (sh.dims[1]) {
    case 16: rc = launch_solo<16>(a, s); break;
    case 32: rc = launch_solo<32>(a, s); break;
    case 64: rc = launch_solo<64>(a, s); break;
    default: return fail(EVO_ERR_UNSUPPORTED, "forage: the hidden width must be 16, 32 or 64");
  }
  if (rc) return rc;
  if (fitness) {
    hipLaunchKernelGGL(world_finish_kernel, dim3((pop + 255) / 256), dim3(256), 0, s, a.reward, pop, worlds, fitness);
    rc = check_launch("world_finish_kernel");
    if (rc) return rc;
  }
  if (reward_out) {
    hipError_t e = hipMemcpyAsync(reward_out, a.reward, static_cast<size_t>(worlds) * pop * sizeof(int32_t),
                                  hipMemcpyDeviceToDevice, s);
    EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "forage: copying the rewards failed: %s", hipGetErrorString(e));
  }
  return EVO_OK;
}

int launch_forage_step(int pop, int worlds, const float* cp, uint64_t seed, uint32_t gen, const float* pos,
                       const float* vel, const uint32_t* counts, const float* actions, float* obs_out, float* pos_out,
                       float* vel_out, int32_t* reward_out, uint32_t* hit_out, hipStream_t s) {
  WorldConst c;
  int rc = fill_const(cp, &c);
  if (rc) return rc;
  const int nb = worlds * c.n_items;
  hipLaunchKernelGGL(world_fill_kernel, dim3((nb + 255) / 256), dim3(256), 0, s, hit_out, nb, 0u);
  rc = check_launch("world_fill_kernel");
  if (rc) return rc;
  StepArgs a;
  a.params = nullptr, a.P = 0, a.pop = pop, a.worlds = worlds;
  a.act[0] = a.act[1] = a.act[2] = EVO_ACT_NONE;
  a.c = c;
  a.key0 = static_cast<uint32_t>(seed), a.key1 = static_cast<uint32_t>(seed >> 32), a.gen = gen, a.gen_dev = nullptr;
  a.pos_in = reinterpret_cast<const float2*>(pos), a.pos_out = reinterpret_cast<float2*>(pos_out);
  a.vel_in = reinterpret_cast<const float2*>(vel), a.vel_out = reinterpret_cast<float2*>(vel_out);
  a.reward = reward_out, a.accumulate = 0;
  a.counts_in = counts, a.hits_prev = nullptr, a.counts_out = nullptr, a.hits_cur = hit_out, a.hits_clear = nullptr;
  a.actions_in = reinterpret_cast<const float2*>(actions), a.obs_out = obs_out;
  return launch_step<16>(a, s);  // the policy is bypassed: any width
}

}  // namespace evo
