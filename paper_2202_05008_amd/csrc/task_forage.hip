// The shared-world task: the whole population lives as agents of one world (Section 3, WaterWorld
// paragraph: every member is spawned in the same task roll-out and measured there).  The paper
// gives the scheme, not the rules; the world is this library's own definition, stated in
// include/evo.h (unit square, food and poison items that reappear elsewhere once eaten, sensing of
// the nearest food, poison and other agent, point-mass motion with drag and walls).
//
// Agents of one world see each other's positions of the current step, so a step is a grid-wide
// dependency: one kernel launch per step, positions double-buffered in the task's workspace.
// A launch is a few microseconds of work spread as widely as its parallelism allows:
//   workgroup = 16 agents x 4 worlds (wave w = world 4 blockIdx.y + w, so the four waves read the
//   same policy weights and the second to fourth find them in the vector cache);
//   four lanes per agent: they split the nearest-neighbour scans (each takes every fourth
//   candidate from LDS, then a four-lane reduction on (distance, index)) and the hidden units of
//   the policy (each a quarter of a layer; the layer's activations go round by lane shuffles).
// Everything that decides an integer -- who is nearest, who touches an item -- is computed in
// binary32 with each operation rounded on its own (no fused multiply-add), as the task defines it.
#include <algorithm>

#include "kernels.h"
#include "philox.h"

namespace evo {

constexpr uint32_t kTagAgent = EVO_TAG_WORLD_AGENT;  // Philox streams of the start positions and of the items
constexpr uint32_t kTagItem = EVO_TAG_WORLD_ITEM;
constexpr int kObs = 8;
constexpr int kAgentsPerBlock = 16;
constexpr int kWorldsPerBlock = 4;

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

// The task's distance: products and sum rounded one by one.
__device__ __forceinline__ float dist2(float dx, float dy) {
#pragma clang fp contract(off)
  const float xx = dx * dx;
  const float yy = dy * dy;
  return xx + yy;
}

struct Nearest {
  float d2, dx, dy;
  int idx;
};

__device__ __forceinline__ void nearest_init(Nearest& n) {
  n.d2 = __builtin_inff(), n.dx = 0.f, n.dy = 0.f, n.idx = 0x7fffffff;
}

// Candidates arrive in increasing index within a lane: strict "<" keeps the lowest index.
__device__ __forceinline__ void nearest_offer(Nearest& n, float2 p, float2 o, int idx) {
  const float dx = o.x - p.x, dy = o.y - p.y;
  const float d2 = dist2(dx, dy);
  if (d2 < n.d2) n.d2 = d2, n.dx = dx, n.dy = dy, n.idx = idx;
}

// Merge over the four lanes of an agent: smaller distance, then lower index.
__device__ __forceinline__ void nearest_quad(Nearest& n) {
#pragma unroll
  for (int m = 1; m <= 2; m <<= 1) {
    const float od = __shfl_xor(n.d2, m), ox = __shfl_xor(n.dx, m), oy = __shfl_xor(n.dy, m);
    const int oi = __shfl_xor(n.idx, m);
    if (od < n.d2 || (od == n.d2 && oi < n.idx)) n.d2 = od, n.dx = ox, n.dy = oy, n.idx = oi;
  }
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

// One dense layer, a quarter of its HO outputs per lane: acc[u] = b[c0 + u] + sum_i in[i] W[i][c0 + u].
template <int HI, int HO>
__device__ __forceinline__ void dense_quarter(const float* __restrict__ W, const float* __restrict__ b, int c0,
                                              const float (&in)[HI], float (&acc)[HO / 4]) {
  constexpr int HQ = HO / 4;
#pragma unroll
  for (int u = 0; u < HQ; u += 2) {
    const float2 bb = *reinterpret_cast<const float2*>(b + c0 + u);
    acc[u] = bb.x, acc[u + 1] = bb.y;
  }
#pragma unroll 8
  for (int i = 0; i < HI; ++i) {
#pragma unroll
    for (int u = 0; u < HQ; u += 2) {
      const float2 w = *reinterpret_cast<const float2*>(W + i * HO + c0 + u);
      acc[u] = fmaf(in[i], w.x, acc[u]);
      acc[u + 1] = fmaf(in[i], w.y, acc[u + 1]);
    }
  }
}

// All HO activations of a layer to every lane of the agent's four.
template <int HO>
__device__ __forceinline__ void gather_quad(const float (&mine)[HO / 4], int lane, float (&full)[HO]) {
  constexpr int HQ = HO / 4;
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int u = 0; u < HQ; ++u) full[s * HQ + u] = __shfl(mine[u], (lane & ~3) | s);
}

// The policy of dims (8, H, H, 2) for one agent; every lane of the four returns both outputs.
template <int H>
__device__ __forceinline__ float2 policy_forward(const float* __restrict__ th, const int (&act)[3], int lane,
                                                 const float (&obs)[kObs]) {
  constexpr int HQ = H / 4;
  const int q = lane & 3, c0 = q * HQ;
  const float* W1 = th;
  const float* b1 = W1 + kObs * H;
  const float* W2 = b1 + H;
  const float* b2 = W2 + H * H;
  const float* W3 = b2 + H;
  const float* b3 = W3 + H * 2;
  float part[HQ], full[H];
  dense_quarter<kObs, H>(W1, b1, c0, obs, part);
#pragma unroll
  for (int u = 0; u < HQ; ++u) part[u] = activate(part[u], act[0]);
  gather_quad<H>(part, lane, full);
  dense_quarter<H, H>(W2, b2, c0, full, part);
#pragma unroll
  for (int u = 0; u < HQ; ++u) part[u] = activate(part[u], act[1]);
  float o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int u = 0; u < HQ; ++u) {
    const float2 w = *reinterpret_cast<const float2*>(W3 + (c0 + u) * 2);
    o0 = fmaf(part[u], w.x, o0);
    o1 = fmaf(part[u], w.y, o1);
  }
  o0 += __shfl_xor(o0, 1), o1 += __shfl_xor(o1, 1);
  o0 += __shfl_xor(o0, 2), o1 += __shfl_xor(o1, 2);
  return make_float2(activate(o0 + b3[0], act[2]), activate(o1 + b3[1], act[2]));
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

template <int H>
__global__ __launch_bounds__(kAgentsPerBlock * 4 * kWorldsPerBlock) void world_step_kernel(StepArgs a) {
  extern __shared__ float2 lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int q = lane & 3;
  const int agent = blockIdx.x * kAgentsPerBlock + (lane >> 2);
  const int world = blockIdx.y * kWorldsPerBlock + wave;
  const bool world_live = world < a.worlds;
  const bool live = world_live && agent < a.pop;
  const int n_items = a.c.n_items;
  float2* s_pos = lds + wave * a.pop;                               // this wave's world: every agent
  float2* s_item = lds + kWorldsPerBlock * a.pop + wave * n_items;  // and every item
  if (a.gen_dev) a.gen = *a.gen_dev;

  if (world_live) {
    const float2* pin = a.pos_in + static_cast<size_t>(world) * a.pop;
    for (int j = lane; j < a.pop; j += 64) s_pos[j] = pin[j];
    for (int i = lane; i < n_items; i += 64) {
      const size_t o = static_cast<size_t>(world) * n_items + i;
      uint32_t cnt = a.counts_in[o];
      if (a.hits_prev) cnt += a.hits_prev[o];
      if (blockIdx.x == 0) {  // one workgroup per world keeps the item book
        if (a.counts_out) a.counts_out[o] = cnt;
        if (a.hits_clear) a.hits_clear[o] = 0u;
      }
      const u32x4 w = philox4x32_10(256u * cnt + static_cast<uint32_t>(i), static_cast<uint32_t>(world), a.gen,
                                    kTagItem, a.key0, a.key1);
      s_item[i] = make_float2(unit_open(w.x), unit_open(w.y));
    }
  }
  __syncthreads();
  if (!live) return;  // no barrier below this line

  const size_t me = static_cast<size_t>(world) * a.pop + agent;
  float2 p = s_pos[agent];
  float2 v = a.vel_in[me];

  Nearest food, poison, other;
  nearest_init(food), nearest_init(poison), nearest_init(other);
  for (int i = q; i < a.c.n_food; i += 4) nearest_offer(food, p, s_item[i], i);
  for (int i = a.c.n_food + q; i < n_items; i += 4) nearest_offer(poison, p, s_item[i], i);
  for (int j = q; j < a.pop; j += 4)
    if (j != agent) nearest_offer(other, p, s_pos[j], j);
  nearest_quad(food), nearest_quad(poison), nearest_quad(other);

  const float obs[kObs] = {v.x, v.y, food.dx, food.dy, poison.dx, poison.dy, other.dx, other.dy};
  if (a.obs_out && q == 0) {
    float4* o = reinterpret_cast<float4*>(a.obs_out + me * kObs);
    o[0] = make_float4(obs[0], obs[1], obs[2], obs[3]);
    o[1] = make_float4(obs[4], obs[5], obs[6], obs[7]);
  }
  float2 action;
  if (a.actions_in)
    action = a.actions_in[me];
  else
    action = policy_forward<H>(a.params + static_cast<size_t>(agent) * a.P, a.act, lane, obs);

  move_axis(a.c, action.x, p.x, v.x);
  move_axis(a.c, action.y, p.y, v.y);

  int reward = 0;
  for (int i = q; i < n_items; i += 4) {
    const float2 it = s_item[i];
    if (dist2(it.x - p.x, it.y - p.y) <= a.c.r2) {
      reward += i < a.c.n_food ? 1 : -1;
      atomicOr(a.hits_cur + static_cast<size_t>(world) * n_items + i, 1u);
    }
  }
  reward += __shfl_xor(reward, 1);
  reward += __shfl_xor(reward, 2);
  if (q == 0) {
    a.pos_out[me] = p;
    a.vel_out[me] = v;
    a.reward[me] = a.accumulate ? a.reward[me] + reward : reward;
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

static size_t step_lds_bytes(int pop, int n_items) {
  return static_cast<size_t>(kWorldsPerBlock) * (pop + n_items) * sizeof(float2);
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

template <int H>
static int launch_step(const StepArgs& a, hipStream_t s) {
  const dim3 grid((a.pop + kAgentsPerBlock - 1) / kAgentsPerBlock, (a.worlds + kWorldsPerBlock - 1) / kWorldsPerBlock);
  hipLaunchKernelGGL(world_step_kernel<H>, grid, dim3(kAgentsPerBlock * 4 * kWorldsPerBlock),
                     step_lds_bytes(a.pop, a.c.n_items), s, a);
  return check_launch("world_step_kernel");
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
  EVO_REQUIRE(step_lds_bytes(pop, c.n_items) <= 65536, EVO_ERR_UNSUPPORTED,
              "forage: at most %d agents per world (positions of four worlds are staged in 64 KB of LDS)",
              65536 / (kWorldsPerBlock * 8) - c.n_items);
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
