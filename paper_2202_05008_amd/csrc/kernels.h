// Launchers shared between the ABI dispatch (rollout.hip) and the kernel files.
#pragma once
#include "common.h"

namespace evo {

struct MlpShape {
  int n_layers;
  int dims[EVO_MAX_LAYERS + 1];
  int act[EVO_MAX_LAYERS];
  int P;
  int max_width;
};

struct ConvShape {
  int H, c1, c2, n_cls, P;
};

enum LossKind { LOSS_NONE = -1, LOSS_CE = 0, LOSS_MSE = 1 };

// Samples per workgroup of the fp32 MLP kernel; one partial loss per (member, tile).
constexpr int kMlpTile = 64;

// fp32 MLP.  loss == LOSS_NONE: writes out[pop][B][A].  Otherwise writes the per-tile loss
// sums partial[pop][tiles] (tiles = ceil(B / kMlpTile)).
int launch_mlp_f32(const MlpShape& sh, const float* params, const float* obs, int64_t obs_stride, int pop, int B,
                   float* out, int loss, const void* target, float* partial, hipStream_t s);

// bf16-weight MLP on the matrix cores; same contract, one workgroup per member.
int mlp_bf16_supported(const MlpShape& sh, int B);
int launch_mlp_bf16(const MlpShape& sh, const uint16_t* params, const float* obs, int64_t obs_stride, int pop, int B,
                    float* out, int loss, const void* target, float* fitness, hipStream_t s);

// ask fused into the bf16 forward: members 2k, 2k+1 of pair k are drawn from (mu, sigma, seed, generation) inside the
// kernel and evaluated together; the population is never written.  Same outputs as launch_mlp_bf16 on what ask stores.
int mlp_bf16_pair_supported(const MlpShape& sh, int B);
int launch_mlp_bf16_pair(const MlpShape& sh, const float* mu, const float* sigma, uint64_t seed, uint32_t gen,
                         const uint32_t* gen_dev, const float* obs, int64_t obs_stride, int pop, int B, float* out,
                         int loss, const void* target, float* fitness, hipStream_t s);

// What the fused calls need of a PGPE state (defined beside the state, in pgpe.hip).
struct PgpeView {
  const float* mu;
  const float* sigma;
  int P;
  uint32_t t;
  const uint32_t* gen_dev;  // the device copy of t, or null
};
int pgpe_view(const pgpe_state* st, PgpeView* out);
int pgpe_check_ask(const pgpe_state* st, int32_t pop, const char* who);
void pgpe_note_ask(pgpe_state* st, uint64_t seed, int32_t pop);

// ask -> forward + loss -> ranks -> tell of an fp32 MLP on a supervised task in one launch (small problems only:
// EVO_ERR_UNSUPPORTED otherwise); the loss sums go through the state's own workspace.
int pgpe_generation_small(pgpe_state* st, uint64_t seed, int32_t pop, const MlpShape& sh, const float* obs,
                          int64_t obs_stride, int B, int loss, const void* target, float scale, float* fitness,
                          hipStream_t s);

// fp32 ConvNet; images shared by all members.  Partials per (member, chunk).  planes_work: convnet_planes_bytes(B)
// bytes of device memory, 16-byte aligned, into which the batch is split into fp16 terms once for all members
// (a small kernel ahead of the members' one); null: every member's workgroups split the images themselves.
int convnet_supported(const ConvShape& sh);
int convnet_chunks(const ConvShape& sh, int pop, int B);
size_t convnet_planes_bytes(int B);
// fitness, scale: with one workgroup per member (chunks == 1) the kernel writes fitness[member] = scale * loss sum itself
// and no partial sums (the caller then skips launch_finalize); ignored otherwise, may be null.
int launch_convnet_f32(const ConvShape& sh, const float* params, const float* images, int pop, int B, float* out,
                       const int32_t* labels, float* partial, int chunks, void* planes_work, float* fitness, float scale,
                       hipStream_t s);

// fitness[m] = scale * sum_j partial[m][j], j in increasing order.
int launch_finalize(const float* partial, int pop, int n, float scale, float* fitness, hipStream_t s);

// fitness[m] = -sum_i (theta[m][i] - x_star[i])^2; partial[pop][sphere_chunks(P)] is scratch.
int sphere_chunks(int P);
int launch_sphere(const void* params, int dtype, const float* x_star, int pop, int P, float* partial, float* fitness,
                  hipStream_t s);

// Fused cart-pole episodes.
int cartpole_supported(const MlpShape& sh, int n_rollouts);
int launch_cartpole(const MlpShape& sh, const float* params, int pop, int n_rollouts, int steps, const float* cp,
                    float init_scale, uint64_t seed, uint32_t gen, const uint32_t* gen_dev, float* fitness, float* ret,
                    float* final_state, float* trace, hipStream_t s);
int launch_cartpole_step(const float* cp, const float* state, const float* action, float* next, float* reward,
                         int n, hipStream_t s);

// The shared-world task: every member is an agent of each of `worlds` worlds; one launch per step.
// `work` holds forage_workspace_bytes(...) bytes.  The state outputs (positions and velocities
// [worlds][pop][2], summed rewards [worlds][pop], times eaten [worlds][items]) may be null.
int forage_supported(const MlpShape& sh, int pop, int worlds, const float* cp);
size_t forage_workspace_bytes(int pop, int worlds, const float* cp);
int launch_forage(const MlpShape& sh, const float* params, int pop, int worlds, int steps, const float* cp,
                  uint64_t seed, uint32_t gen, const uint32_t* gen_dev, void* work, float* fitness, float* pos_out,
                  float* vel_out, int32_t* reward_out, uint32_t* counts_out, hipStream_t s);
int launch_forage_step(int pop, int worlds, const float* cp, uint64_t seed, uint32_t gen, const float* pos,
                       const float* vel, const uint32_t* counts, const float* actions, float* obs_out, float* pos_out,
                       float* vel_out, int32_t* reward_out, uint32_t* hit_out, hipStream_t s);

// The single-agent form: every member alone in its own copy of each world, the whole episode in one launch.
// counts_out is [worlds][pop][items] here.
int forage_solo_supported(const MlpShape& sh, int pop, int worlds, const float* cp);
size_t forage_solo_workspace_bytes(int pop, int worlds);
int launch_forage_solo(const MlpShape& sh, const float* params, int pop, int worlds, int steps, const float* cp,
                       uint64_t seed, uint32_t gen, const uint32_t* gen_dev, void* work, float* fitness, float* pos_out,
                       float* vel_out, int32_t* reward_out, uint32_t* counts_out, hipStream_t s);

// LSTM sequence-to-sequence policy on shared token strings: fitness[pop] = -mean cross-entropy of
// the answer digits and / or logits[pop][B][La][n_out].
int lstm_supported(int V, int H, int n_out, int Lq, int La);
int64_t lstm_param_count(int V, int H, int n_out);
int launch_lstm_seq2seq(int V, int H, int n_out, const float* params, const int32_t* query, const int32_t* answer,
                        int pop, int B, int Lq, int La, float* fitness, float* logits, hipStream_t s);

}  // namespace evo
