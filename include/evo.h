/*
 * evo.h -- C ABI of the MI355X (gfx950) neuroevolution hot path: one PGPE generation on
 * the device for a population in which every member has its own weights.
 *
 * The calls follow the component interfaces the EvoJAX paper describes in Section 4
 * ("Extending EvoJAX"): the algorithm's ask / tell, the global policy's batched
 * get_actions (here pop_forward) and the vectorised task's reset / step loop (here the
 * fused rollout).  The paper prints no formulae; the arithmetic is stated next to each
 * call.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the CALLER.  The library never
 *     allocates, frees or retains device memory, never synchronises (the two checkpoint calls
 *     excepted), and enqueues all work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).
 *   - Pointers without the suffix are host memory, read during the call only.
 *   - Return value: EVO_OK (0) or a negative evo_err.  evo_last_error() gives a
 *     thread-local message for the last failure.  No C++ exception crosses the boundary.
 *   - Notation: pop members, N = pop/2 antithetic pairs, P parameters per member,
 *     generation index t >= 1.  Member m belongs to pair k = m >> 1 with sign +1 (m even)
 *     or -1 (m odd).
 *   - Arrays are dense, row-major, without padding: params[pop][P], obs[pop][B][D],
 *     out[pop][B][A], fitness[pop].  Device pointers must be 16-byte aligned.
 */
#ifndef EVO_GFX950_H
#define EVO_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EVO_OK = 0,
  EVO_ERR_ARG = -1,         /* null pointer, odd or out-of-range pop, bad enum value      */
  EVO_ERR_STATE = -2,       /* tell without a pending ask                                   */
  EVO_ERR_UNSUPPORTED = -3, /* a shape outside the limits of the kernels                    */
  EVO_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed                   */
} evo_err;

enum { EVO_F32 = 0, EVO_BF16 = 1 };                                   /* parameter storage  */
enum { EVO_ACT_NONE = 0, EVO_ACT_TANH = 1, EVO_ACT_RELU = 2 };
enum { EVO_POLICY_MLP = 0, EVO_POLICY_CONVNET = 1, EVO_POLICY_LSTM_SEQ2SEQ = 2 };
enum { EVO_TASK_CLASSIFY = 0, EVO_TASK_REGRESS = 1, EVO_TASK_CARTPOLE = 2, EVO_TASK_SPHERE = 3, EVO_TASK_SEQ2SEQ = 4,
       EVO_TASK_FORAGE = 5, EVO_TASK_FORAGE_SOLO = 6 };
enum { EVO_TAG_NOISE = 0, EVO_TAG_RESET = 1, EVO_TAG_WORLD_AGENT = 2, EVO_TAG_WORLD_ITEM = 3 }; /* Philox stream tags */
enum { EVO_OPT_ADAM = 0, EVO_OPT_CLIPUP = 1, EVO_OPT_MOMENTUM = 2 };  /* optimizer of mu    */
#define EVO_POP_MAX 4096
#define EVO_MAX_LAYERS 8

/* ------------------------------------------------------------------------------------
 * PGPE: the neuroevolution algorithm behind ask / tell (Section 4, "Devising New
 * Algorithms"; PGPE is the algorithm named in Section 5; its gradient estimate is fed to a
 * deep-learning optimizer as Section 2, "Modern ML Optimizers", describes).
 *
 * Noise.  z_k[i] is never stored: both ask and tell regenerate it from the counter-based
 * generator Philox4x32-10 with counter (i >> 2, k, t, EVO_TAG_NOISE) and key
 * (seed & 0xffffffff, seed >> 32).  Word x -> u = (2 (x >> 9) + 1) 2^-24; Box-Muller:
 * words (x0,x1) give z[4j] = r cos(2 pi u1), z[4j+1] = r sin(2 pi u1) with
 * r = sqrt(-2 ln u0); words (x2,x3) give z[4j+2], z[4j+3] the same way.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t P;                /* parameters per member, >= 1                                  */
  int32_t pop_max;          /* largest pop that will be asked, even, <= EVO_POP_MAX         */
  float sigma_init;         /* initial standard deviation of every parameter                */
  float lr_mu;              /* Adam step size for the centre mu                             */
  float lr_sigma;           /* step size for sigma                                          */
  float sigma_max_change;   /* rule 0: |delta sigma| <= sigma_max_change * sigma            */
  float beta1, beta2, eps;  /* Adam constants                                               */
  int32_t sigma_rule;       /* 0 = clipped ascent, 1 = Adam on sigma                        */
  int32_t shaping;          /* 1 = centered ranks, 0 = raw fitness                          */
  int32_t optimizer;        /* update of mu: EVO_OPT_ADAM, EVO_OPT_CLIPUP or EVO_OPT_MOMENTUM */
  float momentum;           /* ClipUp / momentum ascent                                     */
  float max_speed;          /* ClipUp: bound on the Euclidean norm of the velocity, > 0     */
} pgpe_config;

/* The customary values [not in the paper]: sigma_init 0.1, lr_mu 0.01, lr_sigma 0.1, sigma_max_change 0.2,
 * Adam 0.9 / 0.999 / 1e-8, clipped-ascent sigma rule, centered ranks, Adam on mu, momentum 0.9 and, for
 * ClipUp, max_speed = pgpe_clipup_default_max_speed(lr_mu) = 2 lr_mu. */
int pgpe_config_defaults(pgpe_config* cfg, int32_t P, int32_t pop_max);
float pgpe_clipup_default_max_speed(float lr_mu);

typedef struct pgpe_state pgpe_state; /* host handle: config, t, pending (seed, pop), pointers */

/* Bytes of device workspace a state needs (ranks, shaped fitness, norms, the device copy of t). */
size_t pgpe_workspace_bytes(const pgpe_config* cfg);

/* Create a host handle around caller-owned device arrays mu, sigma, m, v (fp32[P] each),
 * aux (fp32[2P]: Adam moments of sigma; required iff sigma_rule == 1, else may be NULL) and
 * work (pgpe_workspace_bytes(cfg) bytes).  Touches no device memory; t starts at 1.
 * The arrays must outlive the handle.  Errors: EVO_ERR_ARG. */
int pgpe_create(pgpe_state** out, const pgpe_config* cfg, float* mu_dev, float* sigma_dev, float* m_dev,
                float* v_dev, float* aux_dev, void* work_dev);
int pgpe_destroy(pgpe_state* st);

/* sigma <- sigma_init, m = v = aux = 0, t <- 1, pending ask dropped.  mu is left as the
 * caller set it (the initial centre is an input). */
int pgpe_reset(pgpe_state* st, void* stream);

/* Generation index t of the next ask (1 after create/reset; +1 per tell); set it to resume. */
int pgpe_get_generation(const pgpe_state* st, uint32_t* t_out);
int pgpe_set_generation(pgpe_state* st, uint32_t t);

/* The centre without perturbation, for testing the current solution (the trainer's "testing" of
 * Section 2): params_dev[r][i] = mu[i] for r < rows, as fp32 or bfloat16 (nearest even).
 * Errors: EVO_ERR_ARG (null, rows outside [1, EVO_POP_MAX], bad dtype), EVO_ERR_HIP. */
int pgpe_center(const pgpe_state* st, int32_t rows, void* params_dev, int32_t dtype, void* stream);

/* Checkpoint (the trainer's periodic model saving, Section 2).  The state of the algorithm is
 * (config, t, mu, sigma, moments): the noise needs no generator state beyond (seed, t), so a run
 * resumed from an exported state continues bit-for-bit.  pgpe_state_export writes a header and the
 * arrays into host_buf (HOST memory, pgpe_state_bytes(st) bytes); pgpe_state_import loads such a
 * buffer into the arrays of a handle created with the same P and sigma_rule and sets t.  Unlike
 * every other call, both wait for `stream` before they return.
 * Errors: EVO_ERR_ARG (null, short buffer, foreign or mismatched state), EVO_ERR_STATE (export
 * while an ask is pending), EVO_ERR_HIP. */
size_t pgpe_state_bytes(const pgpe_state* st);
int pgpe_state_export(const pgpe_state* st, void* host_buf, size_t bytes, void* stream);
int pgpe_state_import(pgpe_state* st, const void* host_buf, size_t bytes, void* stream);

/* Generation index on the device, for callers that record one generation (ask, rollout, tell) in a
 * HIP graph and replay it: kernel arguments are frozen in a graph, so t must not be one.  After this
 * call the state also keeps t in its workspace (*gen_dev_out points at it), ask / tell / ask_sphere
 * read it there, tell advances it with a one-thread kernel in stream order, and Adam's bias
 * corrections are formed in the kernel (same double-precision formula).  Every replay of a captured
 * generation is then the next generation.  The host copy keeps following direct calls;
 * pgpe_sync_generation brings it up to date after replays (it waits for the stream), and
 * pgpe_state_export reads the device copy.  pgpe_set_generation is refused in this mode.
 * Errors: EVO_ERR_ARG, EVO_ERR_STATE (an ask is pending), EVO_ERR_HIP. */
int pgpe_device_generation(pgpe_state* st, const uint32_t** gen_dev_out, void* stream);
int pgpe_sync_generation(pgpe_state* st, void* stream);

/* ask: theta[2k][i] = mu[i] + sigma[i] z_k[i],  theta[2k+1][i] = mu[i] - sigma[i] z_k[i],
 * written to params_dev[pop][P] as fp32 (EVO_F32) or bfloat16 rounded to nearest even
 * (EVO_BF16).  Records (seed, pop) as the pending ask.
 * Errors: EVO_ERR_ARG (null, pop odd / <= 0 / > pop_max, bad dtype), EVO_ERR_HIP. */
int pgpe_ask(pgpe_state* st, uint64_t seed, int32_t pop, void* params_dev, int32_t dtype, void* stream);

/* tell: consumes fitness_dev[pop] (fp32, larger is better) of the pending ask.
 *   ranks   r_m = position of (fitness_m, m) in ascending order (ties -> lower index first;
 *           -0 counts as +0; NaN ranks lowest);  c_m = (2 r_m - (pop-1)) / (2 (pop-1));
 *           with shaping == 0, c_m = fitness_m.
 *   pairs   b = mean(c);  w_k = (c[2k] - c[2k+1]) / 2;  u_k = (c[2k] + c[2k+1]) / 2 - b
 *   grads   g_mu[i] = sigma[i] / N sum_k w_k z_k[i];  g_sigma[i] = sigma[i] / N sum_k u_k (z_k[i]^2 - 1)
 *   update  mu, by cfg.optimizer (the velocity of ClipUp and of momentum ascent lives in m; ClipUp
 *           also uses v as scratch):
 *             ADAM      ascent, bias-corrected with t, eps outside the square root;
 *             CLIPUP    (the optimizer cited with PGPE in Section 5) vel = momentum vel +
 *                       lr_mu g_mu / |g_mu|_2 (zero gradient: + 0); if |vel|_2 > max_speed the
 *                       velocity is scaled to that norm; mu += vel;
 *             MOMENTUM  vel = momentum vel + lr_mu g_mu; mu += vel;
 *           sigma: rule 0: sigma += clip(lr_sigma g_sigma, -+ sigma_max_change sigma);
 *                  rule 1: Adam ascent with moments in aux, then sigma = max(sigma, 1e-8);
 *           t <- t + 1, pending ask cleared.
 * Results are deterministic (fixed reduction order, no floating-point atomics).
 * Errors: EVO_ERR_STATE (no pending ask), EVO_ERR_ARG, EVO_ERR_HIP. */
int pgpe_tell(pgpe_state* st, const float* fitness_dev, void* stream);

/* Measured alternatives to "materialise the population, regenerate the noise" (same Section 4
 * ask / tell interface; both give the results of the calls above up to fp32 rounding order).
 *
 * pgpe_ask_sphere: ask fused with the SPHERE fitness of `rollout`, the population never being
 * written: fitness_dev[m] = -sum_i (theta[m][i] - x_star_dev[i])^2 with theta[m][i] the fp32
 * value pgpe_ask would store.  Records the pending ask like pgpe_ask.  work_dev: caller-owned,
 * pgpe_ask_sphere_workspace_bytes(cfg) bytes (partial sums; contents need not be kept).
 * Errors: EVO_ERR_ARG (null, misaligned, bad pop), EVO_ERR_HIP. */
size_t pgpe_ask_sphere_workspace_bytes(const pgpe_config* cfg);
int pgpe_ask_sphere(pgpe_state* st, uint64_t seed, int32_t pop, const float* x_star_dev, float* fitness_dev,
                    void* work_dev, void* stream);

/* pgpe_tell_stored: tell with the perturbations read back from the fp32 population params_dev[pop][P]
 * that the pending pgpe_ask wrote (only its even rows are read) instead of regenerated:
 * eps_k = theta[2k] - mu;  g_mu[i] = 1/N sum_k w_k eps_k[i];
 * g_sigma[i] = 1/N sum_k u_k (eps_k[i]^2 - sigma[i]^2) / sigma[i]  (0 where sigma[i] = 0);
 * ranks, pair weights, optimizer and sigma rule as in pgpe_tell.  The caller guarantees that
 * params_dev still holds what the pending ask wrote.
 * Errors: EVO_ERR_STATE (no pending ask), EVO_ERR_ARG, EVO_ERR_HIP. */
int pgpe_tell_stored(pgpe_state* st, const float* fitness_dev, const float* params_dev, void* stream);

/* ------------------------------------------------------------------------------------
 * Global policy (Section 2, "Global Policy"; Section 4, "Exploring Novel Policy
 * Architectures"): one network definition evaluated for all members, parameters and
 * observations both being data.
 *
 * MLP  (kind EVO_POLICY_MLP): n_layers dense layers, dims[0..n_layers] widths, act[l] after
 *      layer l.  Flat parameters per layer l in order: W_l[in][out] (out contiguous), b_l[out];
 *      h_{l+1} = act_l(h_l W_l + b_l).  dtype EVO_F32: fp32 arithmetic.  dtype EVO_BF16:
 *      bfloat16 parameters, activations rounded to bfloat16 at each layer input, products
 *      accumulated in fp32 on the matrix cores, bias and activation in fp32.
 * ConvNet (kind EVO_POLICY_CONVNET): dims = {H, c1, c2, n_cls}; input images [B][1][H][H];
 *      conv3x3 (zero-padded, stride 1) -> ReLU -> maxpool 2x2/2, twice, then a dense layer.
 *      Flat parameters: W1[3][3][1][c1], b1[c1], W2[3][3][c1][c2], b2[c2],
 *      Wd[(H/4)(H/4)c2][n_cls], bd[n_cls]; dense input flattened (h, w, c), c fastest.
 *      fp32 results for any finite weights and pixels (the convolutions are evaluated on 16-bit
 *      matrix instructions with two-term operand splits whose scales are set at run time); a member
 *      with a non-finite convolution weight, or an image with an infinite pixel, gets NaN logits (a NaN
 *      pixel is not detected: ReLU and pooling are maximum operations, which drop it).
 * LSTM sequence-to-sequence (kind EVO_POLICY_LSTM_SEQ2SEQ; Section 3, "Seq2Seq Learning"; the carried
 *      cells are the policy state of Section 4): dims = {V, H, n_out}, H = 64 or 128, n_out <= V <= 16.
 *      Tokens are integers in [0, V).  LSTM cell, gates i, f, g, o in columns g H + u:
 *        a = Wx[token] + h Wh + b;  c' = sigmoid(a_f) c + sigmoid(a_i) tanh(a_g);  h' = sigmoid(a_o) tanh(c').
 *      The encoder cell starts from h = c = 0 and reads the query; the decoder cell starts from the
 *      encoder's final (h, c) and takes one step per answer position j, its input being token V - 1
 *      for j = 0 and the true answer token j - 1 afterwards; logits_j = h_j Wo + bo.
 *      Flat parameters: enc Wx[V][4H], Wh[H][4H], b[4H]; dec Wx[V][4H], Wh[H][4H], b[4H];
 *      Wo[H][n_out]; bo[n_out].  fp32 results for any finite weights (two-term fp16 operand splits; a
 *      member with a recurrent weight of 15.99 or more is evaluated by a second, slower build of the kernel
 *      that is launched behind the first and scales each group of weights by its own largest magnitude).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t kind;
  int32_t n_layers;                 /* MLP only */
  int32_t dims[EVO_MAX_LAYERS + 1];
  int32_t act[EVO_MAX_LAYERS];
  int32_t dtype;                    /* storage type of params */
} policy_desc;

/* Number of parameters P the description implies, or a negative evo_err. */
int64_t policy_param_count(const policy_desc* pd);

/* out_dev[pop][B][A] (fp32) = policy(params_dev[m], obs of member m) for every member.
 * obs_dev is fp32 [pop][B][D] with obs_member_stride = B*D elements, or one shared batch
 * [B][D] with obs_member_stride = 0 (every member sees identical observations).
 * Errors: EVO_ERR_ARG, EVO_ERR_UNSUPPORTED (widths / shapes beyond kernel limits), EVO_ERR_HIP. */
int pop_forward(const policy_desc* pd, const void* params_dev, const float* obs_dev, int64_t obs_member_stride,
                float* out_dev, int32_t pop, int32_t B, void* stream);

/* ------------------------------------------------------------------------------------
 * Tasks and the fused roll-out (Section 4, "Experimenting with More Tasks": stateless
 * reset(keys) / step; Section 3: supervised problems are single-step tasks, control tasks
 * run a roll-out loop).  fitness_dev[pop] receives, per member:
 *   CLASSIFY  -mean_b CE(softmax(policy(obs_b)), labels[b])        target_dev = int32 labels[B]
 *   REGRESS   -mean_{b,a} (policy(obs_b)[a] - target[m][b][a])^2   target_dev = fp32 [pop][B][A]
 *   SPHERE    -sum_i (theta[m][i] - x_star[i])^2                    target_dev = fp32 x_star[P]; policy may be NULL
 *   SEQ2SEQ   -mean over samples and answer positions of the cross-entropy of the true answer token
 *             under an EVO_POLICY_LSTM_SEQ2SEQ policy; obs_dev = int32 query tokens [B][seq_in]
 *             (passed through the float pointer), target_dev = int32 answer tokens [B][seq_out],
 *             shared by all members (obs_member_stride = 0); seq_in <= 32, seq_out <= 16.
 *   CARTPOLE  mean over n_rollouts of the episode return of the swing-up task below; the whole
 *             episode (policy weights, environment state) stays on chip for all `steps`.  fp32
 *             results for any finite weights (the second hidden layer runs as two-term fp16 products
 *             with run-time scales, like the ConvNet's second convolution).
 * Cart-pole: state (x, x_d, th, th_d), th from upright; cp = {g, m_cart M, m_pole m, length l,
 *   friction b, force scale, dt, x_limit}; F = force_scale * a - b x_d (a = policy output);
 *   D = 4(M+m) - 3 m cos^2 th;  x_dd = [4F + 2 m l th_d^2 sin th - 3 m g sin th cos th] / D;
 *   th_dd = 3 (g sin th - x_dd cos th) / (2 l);  explicit Euler, derivatives at the old state;
 *   observation (x, x_d, cos th, sin th, th_d); step reward cos(th') exp(-x'^2) at the new
 *   state, counted while alive; the episode dies after a step ending with |x'| > x_limit.
 *   Reset of roll-out r: (x, x_d, th - pi, th_d) = init_scale * the four normals of Philox
 *   counter (0, r, generation, EVO_TAG_RESET) under reset_seed: the same for every member.
 *   FORAGE    the multi-agent scheme of Section 3's WaterWorld paragraph: the whole population is
 *             spawned in the same roll-out, member a as agent a of each of n_rollouts worlds, and
 *             fitness = an agent's summed reward, averaged over the worlds.  The paper gives no
 *             rules; this world is the library's own definition:
 *     cp = {dt, thrust, drag, vmax, touch radius, food items F, poison items Q} (F, Q whole numbers,
 *     F + Q <= 256); policy: fp32 MLP of dims {8, H, H, 2}, H in {16, 32, 64}; pop <= about 4800.
 *     World r: the unit square; agent a starts at rest at (u(x0), u(x1)) of Philox counter
 *     (a, r, generation, EVO_TAG_WORLD_AGENT) under reset_seed; item i (i < F food, else poison) that
 *     has been eaten c times lies at (u(x0), u(x1)) of counter (256 c + i, r, generation,
 *     EVO_TAG_WORLD_ITEM); u(x) = (2 (x >> 9) + 1) 2^-24.
 *     Observation: own velocity (2), offset (other - own) to the nearest food, to the nearest poison,
 *     to the nearest other agent (2 each); nearest by d2 = fl(fl(dx dx) + fl(dy dy)), lowest index
 *     among equals.  Action = the two policy outputs clipped to [-1, 1].
 *     Step, per axis, every operation rounded to binary32 on its own:
 *       v' = clip(fl(fl(drag v) + fl(thrust a)), -vmax, vmax);  p' = fl(p + fl(dt v'));
 *       p' < 0: p' = 0, v' = 0;  p' > 1: p' = 1, v' = 0.
 *     Every item (where it lay at the start of the step) with d2(p', item) <= fl(radius radius) is
 *     touched: +1 (food) or -1 (poison) to every agent that touches it; a touched item has been eaten
 *     once more from the next step on.  `steps` launches of one kernel (agents of a world depend on
 *     each other's positions every step); work_dev holds the worlds' state.
 *   FORAGE_SOLO  the single-agent form of the same world (the paragraph's first sentence): every member lives
 *             alone in its own copy of each world, i.e. a FORAGE world with one agent (agent index 0): all
 *             members start at the same place among the same items and part ways through what they eat; the
 *             offset to the nearest other agent is (0, 0).  Same cp, policy and fitness; pop >= 1; the whole
 *             episode is one launch (weights in registers, the member's items in LDS).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t kind;
  int32_t n_rollouts;          /* CARTPOLE: roll-outs per member (1..64); FORAGE(_SOLO): worlds */
  int32_t B;                   /* CLASSIFY / REGRESS: samples per member                     */
  int32_t P;                   /* SPHERE: parameters per member                              */
  uint64_t reset_seed;         /* CARTPOLE, FORAGE                                           */
  uint32_t generation;         /* CARTPOLE, FORAGE: counter word t of the reset stream       */
  int32_t seq_in;              /* SEQ2SEQ: tokens per query                                  */
  const float* obs_dev;        /* CLASSIFY / REGRESS: observations, see pop_forward          */
  int64_t obs_member_stride;
  const void* target_dev;      /* labels / targets / x_star, see above                       */
  float cp[8];                 /* CARTPOLE / FORAGE constants                                */
  float init_scale;            /* CARTPOLE: scale of the reset normals                       */
  int32_t seq_out;             /* SEQ2SEQ: tokens per answer                                 */
  void* work_dev;              /* workspace of rollout_workspace_bytes(...) bytes, or NULL if 0 */
  const uint32_t* generation_dev; /* CARTPOLE, FORAGE: if not NULL, t is read from this device word at run time
                                     (see pgpe_device_generation) instead of `generation`            */
} task_desc;

/* Bytes of device workspace `rollout` needs for this task / policy / pop (may be 0): partial sums of the
 * members' losses and, for the ConvNet, the shared batch converted once for all members (4 KB per image). */
size_t rollout_workspace_bytes(const task_desc* td, const policy_desc* pd, int32_t pop);

/* Evaluate every member: fitness_dev[pop] as defined above.  `steps` is the episode length
 * for CARTPOLE and FORAGE (FORAGE enqueues steps + 2 kernels and keeps the worlds' state in
 * work_dev, so two roll-outs that share a workspace must not overlap; the same holds for the
 * ConvNet, whose converted batch sits there) and must be 1 for the single-step tasks.
 * Errors: EVO_ERR_ARG, EVO_ERR_UNSUPPORTED, EVO_ERR_HIP. */
int rollout(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop, int32_t steps,
            float* fitness_dev, void* stream);

/* ask fused into the evaluation (Section 4's ask feeding Section 2's global policy without the population ever
 * being stored): fitness_dev[m] = what rollout(td, pd, ...) gives on the bfloat16 population that
 * pgpe_ask(st, seed, pop, ..., EVO_BF16) would write -- bit for bit -- for the EVO_TASK_REGRESS task of the bfloat16
 * MLP 64-256-256-16 with at most 64 observations per member.  One workgroup evaluates the two members of an
 * antithetic pair together from one draw of their noise; mu and sigma are read instead of 2 P bytes per member.
 * Records the pending ask like pgpe_ask; tell regenerates the noise as usual.
 * Errors: EVO_ERR_ARG, EVO_ERR_UNSUPPORTED (any other task / policy: use pgpe_ask + rollout), EVO_ERR_HIP. */
int pgpe_ask_rollout(pgpe_state* st, uint64_t seed, int32_t pop, const task_desc* td, const policy_desc* pd,
                     float* fitness_dev, void* stream);

/* One whole generation -- ask, evaluation, ranks, tell (Section 4's ask / tell around Section 2's evaluation of the
 * population) -- in ONE launch, for problems so small that five launches of a few microseconds each are what a
 * generation costs: the supervised tasks EVO_TASK_CLASSIFY / EVO_TASK_REGRESS of an fp32 MLP whose fan-ins are all
 * below 64, at most 8192 parameters and 512 members, optimizer Adam or momentum.  fitness_dev[pop] and the state (mu, sigma, moments,
 * t) end up bit for bit as pgpe_ask, rollout(td, pd, ...) and pgpe_tell would leave them; the population itself is
 * never stored (each workgroup draws its member's parameters into LDS).  td->work_dev is not used (the loss sums
 * go through the state's workspace; at most 4096 (member, tile of 64 samples) pairs).  Inside the kernel the
 * workgroups that update mu and sigma wait, with a bounded spin, until every workgroup has handed over its loss
 * sum; all others exit, so the wait always ends.
 * Errors: EVO_ERR_ARG, EVO_ERR_UNSUPPORTED (any other task, policy, optimizer or size: use the three calls),
 * EVO_ERR_HIP. */
int pgpe_generation(pgpe_state* st, uint64_t seed, int32_t pop, const task_desc* td, const policy_desc* pd,
                    float* fitness_dev, void* stream);

/* rollout for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same evaluation, by the same kernels, as rollout, but the
 * workspace is a fixed array inside the library's device image (EVO_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends) instead of td->work_dev, which is ignored.  Calls no allocating routine.  A task whose
 * rollout_workspace_bytes() exceeds the array is refused with EVO_ERR_UNSUPPORTED before anything is
 * launched.  Every call on a GPU shares that GPU's array (each kernel writes what it later reads; nothing has to
 * start at zero): two calls that overlap on one GPU, on different streams or threads, race.
 * Errors: as rollout, plus EVO_ERR_UNSUPPORTED (workspace beyond the array), EVO_ERR_HIP (symbol lookup). */
#define EVO_STATIC_SCRATCH_BYTES (8u << 20)
size_t rollout_static_scratch_bytes(void);
int rollout_static_scratch(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                           int32_t steps, float* fitness_dev, void* stream);

/* ------------------------------------------------------------------------------------
 * Hooks that expose intermediate results for exact checks.
 * ------------------------------------------------------------------------------------ */
/* Raw Philox words of counters (block0 + n, pair, gen, tag), n < nblocks: out_dev[4*nblocks]. */
int evo_philox_u32(uint64_t seed, uint32_t gen, uint32_t pair, uint32_t block0, uint32_t nblocks, uint32_t tag,
                   uint32_t* out_dev, void* stream);
/* The fp32 standard normals ask/tell derive from those words: out_dev[4*nblocks]. */
int evo_philox_normal(uint64_t seed, uint32_t gen, uint32_t pair, uint32_t block0, uint32_t nblocks, uint32_t tag,
                      float* out_dev, void* stream);
/* Ranks and shaped fitness of tell's first stage: rank_dev[pop] (u32), shaped_dev[pop] (fp32). */
int evo_centered_rank(const float* fitness_dev, int32_t pop, uint32_t* rank_dev, float* shaped_dev, void* stream);
/* The gradient estimate tell would use for the pending ask, without updating anything:
 * gmu_dev[P], gsigma_dev[P].  params_dev NULL: as pgpe_tell (noise regenerated); else as
 * pgpe_tell_stored from that fp32 population.  The pending ask stays pending. */
int evo_pgpe_gradients(pgpe_state* st, const float* fitness_dev, float* gmu_dev, float* gsigma_dev,
                       const float* params_dev, void* stream);
/* One step of every world of a FORAGE task from a given state with given actions (the policy is
 * bypassed): pos_dev, vel_dev, action_dev [worlds][pop][2] fp32, counts_dev [worlds][F+Q] (times each
 * item was eaten) -> obs_dev [worlds][pop][8], next_pos_dev, next_vel_dev, reward_dev [worlds][pop]
 * (int32, this step's reward), hit_dev [worlds][F+Q] (1 = touched in this step).  Reads td->cp,
 * n_rollouts, reset_seed and generation. */
int evo_forage_step(const task_desc* td, int32_t pop, const float* pos_dev, const float* vel_dev,
                    const uint32_t* counts_dev, const float* action_dev, float* obs_dev, float* next_pos_dev,
                    float* next_vel_dev, int32_t* reward_dev, uint32_t* hit_dev, void* stream);
/* State of a FORAGE or FORAGE_SOLO rollout after `steps` steps: positions and velocities [worlds][pop][2],
 * summed rewards [worlds][pop] (int32), times eaten [worlds][F+Q] (FORAGE_SOLO: [worlds][pop][F+Q]); any may
 * be NULL. */
int evo_forage_state(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop, int32_t steps,
                     float* pos_dev, float* vel_dev, int32_t* reward_dev, uint32_t* counts_dev, void* stream);
/* One cart-pole step for n independent (state, action) pairs: state_dev[n][4], action_dev[n]
 * -> next_dev[n][4], reward_dev[n].  Only td->cp is read. */
int evo_task_step(const task_desc* td, const float* state_dev, const float* action_dev, float* next_dev,
                  float* reward_dev, int32_t n, void* stream);
/* Per-roll-out details of a CARTPOLE rollout: ret_dev[pop][n_rollouts] episode returns and
 * final_dev[pop][n_rollouts][4] final states (either may be NULL). */
int evo_rollout_details(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                        int32_t steps, float* ret_dev, float* final_dev, void* stream);

/* What every step of a CARTPOLE rollout actually used (Section 3, "Control Tasks": the roll-out loop
 * itself): trace_dev[pop][n_rollouts][steps][12] fp32, per record
 *   [0..3] the state (x, x_d, th, th_d) the policy saw at step t,
 *   [4]    the policy's linear output (before the last activation), [5] the action,
 *   [6]    the reward of the step (at the new state), [7] alive before the step (1 / 0),
 *   [8]    the return after the step, [9..11] zero;
 * final_dev[pop][n_rollouts][4] (may be NULL) the state after the last step.  The records come from the
 * kernel behind rollout's fitness, compiled with the stores of the records switched on (same source, same
 * arithmetic: the returns at the end of the trace are bit for bit those of evo_rollout_details), so that
 * each step can be checked on its own along the device's trajectory.
 * Errors: EVO_ERR_ARG, EVO_ERR_UNSUPPORTED, EVO_ERR_HIP. */
int evo_rollout_trace(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                      int32_t steps, float* trace_dev, float* final_dev, void* stream);

/* The policy outputs behind pgpe_ask_rollout: out_dev[pop][B][A] as pop_forward gives on the population that
 * pgpe_ask would write for (seed, current generation).  Leaves the state untouched (no pending ask). */
int evo_ask_forward(pgpe_state* st, uint64_t seed, int32_t pop, const policy_desc* pd, const float* obs_dev,
                    int64_t obs_member_stride, float* out_dev, int32_t B, void* stream);

/* Logits of an EVO_TASK_SEQ2SEQ task: logits_dev[pop][B][seq_out][n_out] (fp32). */
int evo_seq2seq_logits(const task_desc* td, const policy_desc* pd, const void* params_dev, int32_t pop,
                       float* logits_dev, void* stream);

/* Rate probe for the benchmark's "measured next to published" peaks (no step of the path uses it): one launch
 * that fills the GPU with waves running `iters` rounds of eight independent instructions of one kind on
 * registers -- kind 0: fp32 vector multiply-add, 1: v_mfma_f32_16x16x32_f16, 2: v_mfma_f32_32x32x16_bf16,
 * 3: v_mfma_f32_16x16x4_f32.  *flop_out (host) receives the floating-point operations the launch performs;
 * the caller times it.  out_dev: one float of device memory (never written in practice). */
int evo_probe_rate(int32_t kind, int32_t iters, double* flop_out, float* out_dev, void* stream);

const char* evo_last_error(void);
/* Library version string, e.g. "evo-gfx950 0.1". */
const char* evo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EVO_GFX950_H */
