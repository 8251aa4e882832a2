// ABI dispatch for the global policy (pop_forward) and the task roll-out (rollout):
// validates the host-side descriptions, then launches the kernels of the matching family.
// Interfaces after Section 4 of the paper: PolicyNetwork.get_actions on batched task states
// and population parameters; VectorizedTask reset / step carried over the roll-out steps.
#include "kernels.h"

#include <mutex>

using namespace evo;

namespace {

int mlp_shape(const policy_desc* pd, MlpShape* sh) {
  EVO_REQUIRE(pd->n_layers >= 1 && pd->n_layers <= EVO_MAX_LAYERS, EVO_ERR_ARG,
              "policy: n_layers must be in [1, %d] (got %d)", EVO_MAX_LAYERS, pd->n_layers);
  sh->n_layers = pd->n_layers;
  long P = 0;
  int mw = 0;
  for (int i = 0; i <= pd->n_layers; ++i) {
    EVO_REQUIRE(pd->dims[i] >= 1 && pd->dims[i] <= 65536, EVO_ERR_ARG, "policy: dims[%d] = %d out of range", i,
                pd->dims[i]);
    sh->dims[i] = pd->dims[i];
    mw = pd->dims[i] > mw ? pd->dims[i] : mw;
  }
  for (int l = 0; l < pd->n_layers; ++l) {
    EVO_REQUIRE(pd->act[l] >= EVO_ACT_NONE && pd->act[l] <= EVO_ACT_RELU, EVO_ERR_ARG, "policy: bad activation %d",
                pd->act[l]);
    sh->act[l] = pd->act[l];
    P += static_cast<long>(pd->dims[l]) * pd->dims[l + 1] + pd->dims[l + 1];
  }
  EVO_REQUIRE(P < (1l << 30), EVO_ERR_UNSUPPORTED, "policy: too many parameters");
  sh->P = static_cast<int>(P);
  sh->max_width = mw;
  return EVO_OK;
}

int conv_shape(const policy_desc* pd, ConvShape* sh) {
  sh->H = pd->dims[0], sh->c1 = pd->dims[1], sh->c2 = pd->dims[2], sh->n_cls = pd->dims[3];
  EVO_REQUIRE(sh->H >= 4 && sh->c1 >= 1 && sh->c2 >= 1 && sh->n_cls >= 1, EVO_ERR_ARG,
              "convnet: dims must be {H, c1, c2, n_cls}, all positive");
  EVO_REQUIRE(sh->H % 4 == 0, EVO_ERR_ARG, "convnet: H must be a multiple of 4 (got %d)", sh->H);
  const int rc = convnet_supported(*sh);  // bounds every dimension, so the count below cannot overflow
  if (rc) return rc;
  const int feat = (sh->H / 4) * (sh->H / 4) * sh->c2;
  sh->P = 9 * sh->c1 + sh->c1 + 9 * sh->c1 * sh->c2 + sh->c2 + feat * sh->n_cls + sh->n_cls;
  return EVO_OK;
}

int check_policy(const policy_desc* pd) {
  EVO_REQUIRE(pd != nullptr, EVO_ERR_ARG, "policy_desc is null");
  EVO_REQUIRE(pd->kind == EVO_POLICY_MLP || pd->kind == EVO_POLICY_CONVNET || pd->kind == EVO_POLICY_LSTM_SEQ2SEQ,
              EVO_ERR_ARG, "policy: bad kind %d", pd->kind);
  EVO_REQUIRE(pd->dtype == EVO_F32 || pd->dtype == EVO_BF16, EVO_ERR_ARG, "policy: bad dtype %d", pd->dtype);
  return EVO_OK;
}

}  // namespace

extern "C" int64_t policy_param_count(const policy_desc* pd) {
  int rc = check_policy(pd);
  if (rc) return rc;
  if (pd->kind == EVO_POLICY_MLP) {
    MlpShape sh;
    rc = mlp_shape(pd, &sh);
    return rc ? rc : sh.P;
  }
  if (pd->kind == EVO_POLICY_LSTM_SEQ2SEQ) {
    EVO_REQUIRE(pd->dims[0] >= 1 && pd->dims[1] >= 1 && pd->dims[2] >= 1 && pd->dims[1] <= 4096 &&
                    pd->dims[0] <= 65536 && pd->dims[2] <= 65536,
                EVO_ERR_ARG, "lstm: dims must be {V, H, n_out}, all positive");
    return lstm_param_count(pd->dims[0], pd->dims[1], pd->dims[2]);
  }
  ConvShape cs;
  rc = conv_shape(pd, &cs);
  return rc ? rc : cs.P;
}

extern "C" int pop_forward(const policy_desc* pd, const void* params_dev, const float* obs_dev,
                           int64_t obs_member_stride, float* out_dev, int32_t pop, int32_t B, void* stream) {
  int rc = check_policy(pd);
  if (rc) return rc;
  EVO_REQUIRE(params_dev && obs_dev && out_dev, EVO_ERR_ARG, "pop_forward: null device pointer");
  EVO_REQUIRE(pop >= 1 && pop <= 65535 && B >= 1, EVO_ERR_ARG, "pop_forward: pop must be in [1,65535], B >= 1");
  EVO_REQUIRE(obs_member_stride >= 0, EVO_ERR_ARG, "pop_forward: negative obs_member_stride");
  EVO_REQUIRE(aligned16(params_dev) && aligned16(obs_dev) && aligned16(out_dev), EVO_ERR_ARG,
              "pop_forward: device pointers must be 16-byte aligned");
  hipStream_t s = as_stream(stream);
  if (pd->kind == EVO_POLICY_MLP) {
    MlpShape sh;
    rc = mlp_shape(pd, &sh);
    if (rc) return rc;
    EVO_REQUIRE(obs_member_stride == 0 || obs_member_stride == static_cast<int64_t>(B) * sh.dims[0], EVO_ERR_ARG,
                "pop_forward: obs_member_stride must be 0 or B*D");
    if (pd->dtype == EVO_F32)
      return launch_mlp_f32(sh, static_cast<const float*>(params_dev), obs_dev, obs_member_stride, pop, B, out_dev,
                            LOSS_NONE, nullptr, nullptr, s);
    rc = mlp_bf16_supported(sh, B);
    if (rc) return rc;
    return launch_mlp_bf16(sh, static_cast<const uint16_t*>(params_dev), obs_dev, obs_member_stride, pop, B, out_dev,
                           LOSS_NONE, nullptr, nullptr, s);
  }
  EVO_REQUIRE(pd->kind != EVO_POLICY_LSTM_SEQ2SEQ, EVO_ERR_UNSUPPORTED,
              "pop_forward: the sequence-to-sequence policy consumes token strings: use rollout or evo_seq2seq_logits");
  ConvShape cs;
  rc = conv_shape(pd, &cs);
  if (rc) return rc;
  EVO_REQUIRE(pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED, "convnet: only fp32 parameters are supported");
  EVO_REQUIRE(obs_member_stride == 0, EVO_ERR_UNSUPPORTED, "convnet: images must be shared (obs_member_stride 0)");
  rc = convnet_supported(cs);
  if (rc) return rc;
  return launch_convnet_f32(cs, static_cast<const float*>(params_dev), obs_dev, pop, B, out_dev, nullptr, nullptr, 0,
                            nullptr, nullptr, 0.f, s);
}

namespace {

// Number of partial sums per member that `rollout` keeps in the workspace.
int partials_per_member(const task_desc* td, const policy_desc* pd, int pop) {
  if (td->kind == EVO_TASK_SPHERE) return td->P >= 1 ? sphere_chunks(td->P) : 0;
  if (td->kind != EVO_TASK_CLASSIFY && td->kind != EVO_TASK_REGRESS) return 0;
  if (pd->kind == EVO_POLICY_LSTM_SEQ2SEQ) return 0;
  if (pd->kind == EVO_POLICY_CONVNET) {
    ConvShape cs;
    if (conv_shape(pd, &cs)) return 0;
    return convnet_chunks(cs, pop, td->B);
  }
  if (pd->dtype == EVO_BF16) return 0;
  return (td->B + kMlpTile - 1) / kMlpTile;
}

// Bytes of the partial sums in the workspace (a multiple of 256), and of what follows them: the ConvNet's batch
// split into fp16 terms once for all members.
size_t partials_bytes(const task_desc* td, const policy_desc* pd, int pop) {
  return (static_cast<size_t>(partials_per_member(td, pd, pop)) * pop * sizeof(float) + 255) & ~size_t(255);
}
size_t planes_bytes(const task_desc* td, const policy_desc* pd) {
  if (td->kind != EVO_TASK_CLASSIFY || pd == nullptr || pd->kind != EVO_POLICY_CONVNET || td->B < 1) return 0;
  return convnet_planes_bytes(td->B);
}

int check_task(const task_desc* td) {
  EVO_REQUIRE(td != nullptr, EVO_ERR_ARG, "task_desc is null");
  EVO_REQUIRE(td->kind >= EVO_TASK_CLASSIFY && td->kind <= EVO_TASK_FORAGE_SOLO, EVO_ERR_ARG, "task: bad kind %d",
              td->kind);
  return EVO_OK;
}

}  // namespace

extern "C" size_t rollout_workspace_bytes(const task_desc* td, const policy_desc* pd, int32_t pop) {
  if (check_task(td) || pop < 1) return 0;
  if (td->kind == EVO_TASK_CARTPOLE || td->kind == EVO_TASK_SEQ2SEQ) return 0;
  if (td->kind == EVO_TASK_FORAGE) return forage_workspace_bytes(pop, td->n_rollouts, td->cp);
  if (td->kind == EVO_TASK_FORAGE_SOLO) return forage_solo_workspace_bytes(pop, td->n_rollouts);
  if (td->kind != EVO_TASK_SPHERE && check_policy(pd)) return 0;
  return partials_bytes(td, pd, pop) + planes_bytes(td, pd);
}

// The sequence-to-sequence task: fitness and / or logits of every member.
static int seq2seq_impl(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                        float* fitness_dev, float* logits_dev, void* stream) {
  int rc = check_policy(pd);
  if (rc) return rc;
  EVO_REQUIRE(pd->kind == EVO_POLICY_LSTM_SEQ2SEQ && pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED,
              "seq2seq: needs an fp32 EVO_POLICY_LSTM_SEQ2SEQ policy");
  EVO_REQUIRE(td->B >= 1 && td->obs_dev && td->target_dev, EVO_ERR_ARG,
              "seq2seq: needs B >= 1, query tokens (obs_dev) and answer tokens (target_dev)");
  EVO_REQUIRE(td->obs_member_stride == 0, EVO_ERR_UNSUPPORTED, "seq2seq: the token strings must be shared");
  const int V = pd->dims[0], H = pd->dims[1], n_out = pd->dims[2];
  rc = lstm_supported(V, H, n_out, td->seq_in, td->seq_out);
  if (rc) return rc;
  return launch_lstm_seq2seq(V, H, n_out, static_cast<const float*>(params_dev),
                             reinterpret_cast<const int32_t*>(td->obs_dev),
                             static_cast<const int32_t*>(td->target_dev), pop, td->B, td->seq_in, td->seq_out,
                             fitness_dev, logits_dev, as_stream(stream));
}

// The shared-world task: fitness and / or the state after the last step.
static int forage_impl(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop, int32_t steps,
                       float* fitness_dev, float* pos_dev, float* vel_dev, int32_t* reward_dev, uint32_t* counts_dev,
                       void* stream) {
  EVO_REQUIRE(td != nullptr && (td->kind == EVO_TASK_FORAGE || td->kind == EVO_TASK_FORAGE_SOLO), EVO_ERR_ARG,
              "forage: needs an EVO_TASK_FORAGE or EVO_TASK_FORAGE_SOLO task");
  const bool solo = td->kind == EVO_TASK_FORAGE_SOLO;
  int rc = check_policy(pd);
  if (rc) return rc;
  EVO_REQUIRE(pd->kind == EVO_POLICY_MLP && pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED,
              "forage: needs an fp32 MLP policy");
  EVO_REQUIRE(params_dev != nullptr && aligned16(params_dev), EVO_ERR_ARG,
              "forage: params_dev must be a 16-byte aligned device pointer");
  EVO_REQUIRE(pop >= (solo ? 1 : 2) && pop <= 65535, EVO_ERR_ARG, "forage: pop must be in [%d,65535] (got %d)",
              solo ? 1 : 2, pop);
  EVO_REQUIRE(steps >= 1 && steps <= (1 << 20), EVO_ERR_ARG, "forage: steps must be in [1, 2^20]");
  EVO_REQUIRE(td->work_dev != nullptr && aligned16(td->work_dev), EVO_ERR_ARG,
              "forage: work_dev must hold rollout_workspace_bytes() bytes, 16-byte aligned");
  MlpShape sh;
  rc = mlp_shape(pd, &sh);
  if (rc) return rc;
  if (solo) {
    rc = forage_solo_supported(sh, pop, td->n_rollouts, td->cp);
    if (rc) return rc;
    return launch_forage_solo(sh, static_cast<const float*>(params_dev), pop, td->n_rollouts, steps, td->cp,
                              td->reset_seed, td->generation, td->generation_dev, td->work_dev, fitness_dev, pos_dev,
                              vel_dev, reward_dev, counts_dev, as_stream(stream));
  }
  rc = forage_supported(sh, pop, td->n_rollouts, td->cp);
  if (rc) return rc;
  return launch_forage(sh, static_cast<const float*>(params_dev), pop, td->n_rollouts, steps, td->cp, td->reset_seed,
                       td->generation, td->generation_dev, td->work_dev, fitness_dev, pos_dev, vel_dev, reward_dev,
                       counts_dev, as_stream(stream));
}

static int rollout_impl(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                        int32_t steps, float* fitness_dev, float* ret_dev, float* final_dev, float* trace_dev,
                        void* stream) {
  int rc = check_task(td);
  if (rc) return rc;
  EVO_REQUIRE(params_dev != nullptr, EVO_ERR_ARG, "rollout: null device pointer");
  EVO_REQUIRE(pop >= 1 && pop <= 65535, EVO_ERR_ARG, "rollout: pop must be in [1,65535] (got %d)", pop);
  EVO_REQUIRE(aligned16(params_dev), EVO_ERR_ARG, "rollout: params_dev must be 16-byte aligned");
  hipStream_t s = as_stream(stream);
  if (td->kind == EVO_TASK_SPHERE) {
    EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout: fitness_dev is null");
    EVO_REQUIRE(steps == 1, EVO_ERR_ARG, "rollout: single-step task needs steps == 1");
    EVO_REQUIRE(td->P >= 1 && td->target_dev != nullptr, EVO_ERR_ARG, "sphere: needs P >= 1 and x_star");
    const int dtype = pd ? pd->dtype : EVO_F32;
    EVO_REQUIRE(dtype == EVO_F32 || dtype == EVO_BF16, EVO_ERR_ARG, "sphere: bad dtype");
    EVO_REQUIRE(td->work_dev != nullptr, EVO_ERR_ARG, "sphere: work_dev is null but rollout_workspace_bytes() > 0");
    EVO_REQUIRE(aligned16(td->target_dev) && aligned16(td->work_dev), EVO_ERR_ARG,
                "sphere: x_star and work_dev must be 16-byte aligned");
    return launch_sphere(params_dev, dtype, static_cast<const float*>(td->target_dev), pop, td->P,
                         static_cast<float*>(td->work_dev), fitness_dev, s);
  }
  if (td->kind == EVO_TASK_FORAGE || td->kind == EVO_TASK_FORAGE_SOLO) {
    EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout: fitness_dev is null");
    return forage_impl(td, pd, params_dev, pop, steps, fitness_dev, nullptr, nullptr, nullptr, nullptr, stream);
  }
  if (td->kind == EVO_TASK_SEQ2SEQ) {
    EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout: fitness_dev is null");
    EVO_REQUIRE(steps == 1, EVO_ERR_ARG, "rollout: the sequence-to-sequence task is a single-step task (steps == 1)");
    return seq2seq_impl(td, pd, params_dev, pop, fitness_dev, nullptr, stream);
  }
  rc = check_policy(pd);
  if (rc) return rc;
  if (td->kind == EVO_TASK_CARTPOLE) {
    EVO_REQUIRE(pd->kind == EVO_POLICY_MLP && pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED,
                "cartpole: needs an fp32 MLP policy");
    EVO_REQUIRE(steps >= 1 && steps <= (1 << 24), EVO_ERR_ARG, "cartpole: steps out of range");
    EVO_REQUIRE(fitness_dev || ret_dev || final_dev || trace_dev, EVO_ERR_ARG, "cartpole: no output requested");
    MlpShape sh;
    rc = mlp_shape(pd, &sh);
    if (rc) return rc;
    rc = cartpole_supported(sh, td->n_rollouts);
    if (rc) return rc;
    return launch_cartpole(sh, static_cast<const float*>(params_dev), pop, td->n_rollouts, steps, td->cp,
                           td->init_scale, td->reset_seed, td->generation, td->generation_dev, fitness_dev, ret_dev,
                           final_dev, trace_dev, s);
  }
  // supervised single-step tasks
  EVO_REQUIRE(pd->kind != EVO_POLICY_LSTM_SEQ2SEQ, EVO_ERR_UNSUPPORTED,
              "rollout: the sequence-to-sequence policy needs the EVO_TASK_SEQ2SEQ task");
  EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout: fitness_dev is null");
  EVO_REQUIRE(steps == 1, EVO_ERR_ARG, "rollout: single-step task needs steps == 1");
  EVO_REQUIRE(td->B >= 1 && td->obs_dev && td->target_dev, EVO_ERR_ARG, "rollout: needs B >= 1, obs and targets");
  EVO_REQUIRE(td->obs_member_stride >= 0, EVO_ERR_ARG, "rollout: negative obs_member_stride");
  EVO_REQUIRE(aligned16(td->obs_dev) && aligned16(td->target_dev), EVO_ERR_ARG,
              "rollout: obs and target must be 16-byte aligned");
  const int loss = td->kind == EVO_TASK_CLASSIFY ? LOSS_CE : LOSS_MSE;
  const int n_part = partials_per_member(td, pd, pop);
  EVO_REQUIRE(n_part == 0 || td->work_dev != nullptr, EVO_ERR_ARG,
              "rollout: work_dev is null but rollout_workspace_bytes() > 0");
  float* partial = static_cast<float*>(td->work_dev);
  if (pd->kind == EVO_POLICY_CONVNET) {
    EVO_REQUIRE(loss == LOSS_CE, EVO_ERR_UNSUPPORTED, "convnet: only the classification task is supported");
    EVO_REQUIRE(pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED, "convnet: only fp32 parameters are supported");
    EVO_REQUIRE(td->obs_member_stride == 0, EVO_ERR_UNSUPPORTED, "convnet: images must be shared");
    EVO_REQUIRE(aligned16(td->work_dev), EVO_ERR_ARG, "convnet: work_dev must be 16-byte aligned");
    ConvShape cs;
    rc = conv_shape(pd, &cs);
    if (rc) return rc;
    rc = convnet_supported(cs);
    if (rc) return rc;
    rc = launch_convnet_f32(cs, static_cast<const float*>(params_dev), td->obs_dev, pop, td->B, nullptr,
                            static_cast<const int32_t*>(td->target_dev), partial, n_part,
                            static_cast<unsigned char*>(td->work_dev) + partials_bytes(td, pd, pop), fitness_dev,
                            -1.0f / static_cast<float>(td->B), s);
    if (rc || n_part == 1) return rc;  // one workgroup per member: the kernel has written the fitness itself
    return launch_finalize(partial, pop, n_part, -1.0f / static_cast<float>(td->B), fitness_dev, s);
  }
  MlpShape sh;
  rc = mlp_shape(pd, &sh);
  if (rc) return rc;
  EVO_REQUIRE(td->obs_member_stride == 0 || td->obs_member_stride == static_cast<int64_t>(td->B) * sh.dims[0],
              EVO_ERR_ARG, "rollout: obs_member_stride must be 0 or B*D");
  const int A = sh.dims[sh.n_layers];
  if (pd->dtype == EVO_BF16) {
    rc = mlp_bf16_supported(sh, td->B);
    if (rc) return rc;
    return launch_mlp_bf16(sh, static_cast<const uint16_t*>(params_dev), td->obs_dev, td->obs_member_stride, pop,
                           td->B, nullptr, loss, td->target_dev, fitness_dev, s);
  }
  rc = launch_mlp_f32(sh, static_cast<const float*>(params_dev), td->obs_dev, td->obs_member_stride, pop, td->B,
                      nullptr, loss, td->target_dev, partial, s);
  if (rc) return rc;
  const float scale = loss == LOSS_CE ? -1.0f / static_cast<float>(td->B)
                                      : -1.0f / (static_cast<float>(td->B) * static_cast<float>(A));
  return launch_finalize(partial, pop, n_part, scale, fitness_dev, s);
}

extern "C" int rollout(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                       int32_t steps, float* fitness_dev, void* stream) {
  EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout: fitness_dev is null");
  return rollout_impl(td, pd, params_dev, pop, steps, fitness_dev, nullptr, nullptr, nullptr, stream);
}

// ---- ask fused into the evaluation: the population is never written ---------------------------------------
static int ask_forward_impl(pgpe_state* st, uint64_t seed, int32_t pop, const policy_desc* pd, const float* obs_dev,
                            int64_t obs_member_stride, int32_t B, float* out_dev, int loss, const void* target_dev,
                            float* fitness_dev, const char* who, void* stream) {
  PgpeView v;
  int rc = pgpe_view(st, &v);
  if (rc) return rc;
  rc = pgpe_check_ask(st, pop, who);
  if (rc) return rc;
  rc = check_policy(pd);
  if (rc) return rc;
  EVO_REQUIRE(pd->kind == EVO_POLICY_MLP && pd->dtype == EVO_BF16, EVO_ERR_UNSUPPORTED,
              "%s: needs a bfloat16 MLP policy", who);
  MlpShape sh;
  rc = mlp_shape(pd, &sh);
  if (rc) return rc;
  EVO_REQUIRE(sh.P == v.P, EVO_ERR_ARG, "%s: the policy has %d parameters, the PGPE state %d", who, sh.P, v.P);
  EVO_REQUIRE(B >= 1 && obs_dev != nullptr && aligned16(obs_dev), EVO_ERR_ARG,
              "%s: needs B >= 1 and 16-byte aligned observations", who);
  EVO_REQUIRE(obs_member_stride == 0 || obs_member_stride == static_cast<int64_t>(B) * sh.dims[0], EVO_ERR_ARG,
              "%s: obs_member_stride must be 0 or B*D", who);
  rc = mlp_bf16_pair_supported(sh, B);
  if (rc) return rc;
  return launch_mlp_bf16_pair(sh, v.mu, v.sigma, seed, v.t, v.gen_dev, obs_dev, obs_member_stride, pop, B, out_dev, loss,
                              target_dev, fitness_dev, as_stream(stream));
}

extern "C" int pgpe_ask_rollout(pgpe_state* st, uint64_t seed, int32_t pop, const task_desc* td, const policy_desc* pd,
                                float* fitness_dev, void* stream) {
  EVO_REQUIRE(st != nullptr && fitness_dev != nullptr, EVO_ERR_ARG, "pgpe_ask_rollout: null argument");
  int rc = check_task(td);
  if (rc) return rc;
  EVO_REQUIRE(td->kind == EVO_TASK_REGRESS, EVO_ERR_UNSUPPORTED,
              "pgpe_ask_rollout: only the regression task of a bfloat16 MLP is fused (the sphere: pgpe_ask_sphere)");
  EVO_REQUIRE(td->target_dev != nullptr && aligned16(td->target_dev), EVO_ERR_ARG,
              "pgpe_ask_rollout: needs 16-byte aligned targets");
  rc = ask_forward_impl(st, seed, pop, pd, td->obs_dev, td->obs_member_stride, td->B, nullptr, LOSS_MSE, td->target_dev,
                        fitness_dev, "pgpe_ask_rollout", stream);
  if (rc) return rc;
  pgpe_note_ask(st, seed, pop);
  return EVO_OK;
}

extern "C" int pgpe_generation(pgpe_state* st, uint64_t seed, int32_t pop, const task_desc* td, const policy_desc* pd,
                               float* fitness_dev, void* stream) {
  EVO_REQUIRE(st != nullptr && fitness_dev != nullptr, EVO_ERR_ARG, "pgpe_generation: null argument");
  int rc = check_task(td);
  if (rc) return rc;
  EVO_REQUIRE(td->kind == EVO_TASK_CLASSIFY || td->kind == EVO_TASK_REGRESS, EVO_ERR_UNSUPPORTED,
              "pgpe_generation: only the supervised tasks of an fp32 MLP run as one launch");
  EVO_REQUIRE(pd != nullptr && pd->kind == EVO_POLICY_MLP && pd->dtype == EVO_F32, EVO_ERR_UNSUPPORTED,
              "pgpe_generation: only the supervised tasks of an fp32 MLP run as one launch");
  EVO_REQUIRE(td->B >= 1 && td->obs_dev != nullptr && td->target_dev != nullptr, EVO_ERR_ARG,
              "pgpe_generation: B >= 1, obs_dev and target_dev required");
  EVO_REQUIRE(td->obs_member_stride >= 0, EVO_ERR_ARG, "pgpe_generation: negative obs_member_stride");
  EVO_REQUIRE(aligned16(td->obs_dev) && aligned16(td->target_dev), EVO_ERR_ARG,
              "pgpe_generation: obs and target must be 16-byte aligned");
  MlpShape sh;
  rc = mlp_shape(pd, &sh);
  if (rc) return rc;
  EVO_REQUIRE(td->obs_member_stride == 0 || td->obs_member_stride == static_cast<int64_t>(td->B) * sh.dims[0],
              EVO_ERR_ARG, "pgpe_generation: obs_member_stride must be 0 or B*D");
  bool narrow = true;  // the vector-ALU forward: every fan-in below 64
  for (int l = 0; l < sh.n_layers; ++l) narrow = narrow && sh.dims[l] < 64;
  EVO_REQUIRE(narrow, EVO_ERR_UNSUPPORTED, "pgpe_generation: networks with a fan-in of 64 or more take ask, rollout, tell");
  const int loss = td->kind == EVO_TASK_CLASSIFY ? LOSS_CE : LOSS_MSE;
  const int A = sh.dims[sh.n_layers];
  const float scale = loss == LOSS_CE ? -1.0f / static_cast<float>(td->B)
                                      : -1.0f / (static_cast<float>(td->B) * static_cast<float>(A));
  return pgpe_generation_small(st, seed, pop, sh, td->obs_dev, td->obs_member_stride, td->B, loss, td->target_dev, scale,
                               fitness_dev, as_stream(stream));
}

extern "C" int evo_ask_forward(pgpe_state* st, uint64_t seed, int32_t pop, const policy_desc* pd, const float* obs_dev,
                               int64_t obs_member_stride, float* out_dev, int32_t B, void* stream) {
  EVO_REQUIRE(st != nullptr && out_dev != nullptr && aligned16(out_dev), EVO_ERR_ARG,
              "evo_ask_forward: needs a state and a 16-byte aligned output");
  return ask_forward_impl(st, seed, pop, pd, obs_dev, obs_member_stride, B, out_dev, LOSS_NONE, nullptr, nullptr,
                          "evo_ask_forward", stream);
}

// ---- rollout for callers that cannot allocate: the workspace lives in the library's image ----------
// `scratch` is a host-side stand-in for the device array, not an address: kernels are given the address
// that hipGetSymbolAddress returns for the device that is current, looked up once per device.
constexpr size_t kStaticScratchBytes = EVO_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // per device: where its copy of `scratch` lives

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  EVO_REQUIRE(e == hipSuccess, EVO_ERR_HIP, "rollout_static_scratch: hipGetDevice failed: %s", hipGetErrorString(e));
  EVO_REQUIRE(dev >= 0 && dev < kMaxDevices, EVO_ERR_UNSUPPORTED, "rollout_static_scratch: device index %d beyond %d",
              dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) (void)hipGetLastError();
    EVO_REQUIRE(e == hipSuccess && p != nullptr, EVO_ERR_HIP, "rollout_static_scratch: hipGetSymbolAddress failed: %s",
                hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return EVO_OK;
}

}  // namespace

extern "C" size_t rollout_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int rollout_static_scratch(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                                      int32_t steps, float* fitness_dev, void* stream) {
  EVO_REQUIRE(fitness_dev != nullptr, EVO_ERR_ARG, "rollout_static_scratch: fitness_dev is null");
  int rc = check_task(td);
  if (rc) return rc;
  EVO_REQUIRE(pop >= 1 && pop <= 65535, EVO_ERR_ARG, "rollout_static_scratch: pop must be in [1,65535] (got %d)", pop);
  const size_t need = rollout_workspace_bytes(td, pd, pop);
  EVO_REQUIRE(need <= kStaticScratchBytes, EVO_ERR_UNSUPPORTED,
              "rollout_static_scratch: this task needs %zu bytes of workspace, the built-in scratch holds %zu: "
              "use rollout with a caller-owned workspace",
              need, kStaticScratchBytes);
  task_desc local = *td;
  void* ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc) return rc;
  local.work_dev = need ? ptr : nullptr;
  return rollout_impl(&local, pd, params_dev, pop, steps, fitness_dev, nullptr, nullptr, nullptr, stream);
}

extern "C" int evo_rollout_details(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                                   int32_t steps, float* ret_dev, float* final_dev, void* stream) {
  EVO_REQUIRE(td != nullptr && td->kind == EVO_TASK_CARTPOLE, EVO_ERR_ARG,
              "evo_rollout_details: only the cart-pole task has per-roll-out details");
  EVO_REQUIRE(ret_dev || final_dev, EVO_ERR_ARG, "evo_rollout_details: no output requested");
  return rollout_impl(td, pd, params_dev, pop, steps, nullptr, ret_dev, final_dev, nullptr, stream);
}

extern "C" int evo_rollout_trace(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                                 int32_t steps, float* trace_dev, float* final_dev, void* stream) {
  EVO_REQUIRE(td != nullptr && td->kind == EVO_TASK_CARTPOLE, EVO_ERR_ARG,
              "evo_rollout_trace: only the cart-pole task records a trace");
  EVO_REQUIRE(trace_dev != nullptr && aligned16(trace_dev), EVO_ERR_ARG,
              "evo_rollout_trace: trace_dev must be a 16-byte aligned device pointer");
  return rollout_impl(td, pd, params_dev, pop, steps, nullptr, nullptr, final_dev, trace_dev, stream);
}

extern "C" int evo_seq2seq_logits(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                                  float* logits_dev, void* stream) {
  EVO_REQUIRE(td != nullptr && td->kind == EVO_TASK_SEQ2SEQ, EVO_ERR_ARG,
              "evo_seq2seq_logits: needs an EVO_TASK_SEQ2SEQ task");
  EVO_REQUIRE(params_dev && logits_dev, EVO_ERR_ARG, "evo_seq2seq_logits: null device pointer");
  EVO_REQUIRE(pop >= 1 && pop <= 65535, EVO_ERR_ARG, "evo_seq2seq_logits: pop must be in [1,65535] (got %d)", pop);
  EVO_REQUIRE(aligned16(params_dev), EVO_ERR_ARG, "evo_seq2seq_logits: params_dev must be 16-byte aligned");
  return seq2seq_impl(td, pd, params_dev, pop, nullptr, logits_dev, stream);
}

extern "C" int evo_forage_state(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                                int32_t steps, float* pos_dev, float* vel_dev, int32_t* reward_dev,
                                uint32_t* counts_dev, void* stream) {
  EVO_REQUIRE(pos_dev || vel_dev || reward_dev || counts_dev, EVO_ERR_ARG, "evo_forage_state: no output requested");
  return forage_impl(td, pd, params_dev, pop, steps, nullptr, pos_dev, vel_dev, reward_dev, counts_dev, stream);
}

extern "C" int evo_forage_step(const task_desc* td, int32_t pop, const float* pos_dev, const float* vel_dev,
                               const uint32_t* counts_dev, const float* action_dev, float* obs_dev, float* next_pos_dev,
                               float* next_vel_dev, int32_t* reward_dev, uint32_t* hit_dev, void* stream) {
  EVO_REQUIRE(td != nullptr && td->kind == EVO_TASK_FORAGE, EVO_ERR_ARG, "evo_forage_step: needs an EVO_TASK_FORAGE task");
  EVO_REQUIRE(pos_dev && vel_dev && counts_dev && action_dev && obs_dev && next_pos_dev && next_vel_dev &&
                  reward_dev && hit_dev,
              EVO_ERR_ARG, "evo_forage_step: null device pointer");
  EVO_REQUIRE(aligned16(obs_dev) && aligned16(pos_dev) && aligned16(vel_dev) && aligned16(action_dev) &&
                  aligned16(next_pos_dev) && aligned16(next_vel_dev),
              EVO_ERR_ARG, "evo_forage_step: device pointers must be 16-byte aligned");
  EVO_REQUIRE(pop >= 2 && pop <= 65535, EVO_ERR_ARG, "evo_forage_step: pop must be in [2,65535] (got %d)", pop);
  MlpShape any;
  any.n_layers = 3, any.dims[0] = 8, any.dims[1] = any.dims[2] = 16, any.dims[3] = 2, any.P = 450;
  int rc = forage_supported(any, pop, td->n_rollouts, td->cp);
  if (rc) return rc;
  return launch_forage_step(pop, td->n_rollouts, td->cp, td->reset_seed, td->generation, pos_dev, vel_dev, counts_dev,
                            action_dev, obs_dev, next_pos_dev, next_vel_dev, reward_dev, hit_dev, as_stream(stream));
}

extern "C" int evo_task_step(const task_desc* td, const float* state_dev, const float* action_dev, float* next_dev,
                             float* reward_dev, int32_t n, void* stream) {
  EVO_REQUIRE(td && state_dev && action_dev && next_dev && reward_dev, EVO_ERR_ARG, "evo_task_step: null argument");
  EVO_REQUIRE(n >= 0, EVO_ERR_ARG, "evo_task_step: negative n");
  if (n == 0) return EVO_OK;
  return launch_cartpole_step(td->cp, state_dev, action_dev, next_dev, reward_dev, n, as_stream(stream));
}
