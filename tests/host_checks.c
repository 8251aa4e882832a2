/* Host-side paths of the C ABI, called from plain C without a GPU: defaults, descriptor validation, size
 * queries, the argument checks that come before any launch, create / destroy.  Built by
 * tests/test_host_sanitizers_cpu.py together with the library's sources, host code under AddressSanitizer and
 * UndefinedBehaviorSanitizer; exit status 0 = every check held and no sanitizer report. */
#include <stdio.h>
#include <string.h>
#include "evo.h"

static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "host_checks.c:%d: %s failed (last error: %s)\n", __LINE__, #cond, evo_last_error()); \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

int main(void) {
  void* fake = (void*)0x1000; /* never dereferenced on the host */
  pgpe_config cfg;
  CHECK(strncmp(evo_version(), "evo-gfx950", 10) == 0);
  CHECK(pgpe_config_defaults(&cfg, 676, 64) == EVO_OK);
  CHECK(cfg.P == 676 && cfg.pop_max == 64 && cfg.sigma_init > 0.f && cfg.optimizer == EVO_OPT_ADAM);
  CHECK(pgpe_config_defaults(NULL, 676, 64) == EVO_ERR_ARG);
  CHECK(pgpe_clipup_default_max_speed(0.15f) > 0.f);
  CHECK(pgpe_workspace_bytes(&cfg) >= 64 * 12);
  CHECK(pgpe_ask_sphere_workspace_bytes(&cfg) > 0);
  CHECK(rollout_static_scratch_bytes() == EVO_STATIC_SCRATCH_BYTES);

  pgpe_config bad = cfg;
  bad.pop_max = 63;
  CHECK(pgpe_workspace_bytes(&bad) == 0);
  bad = cfg;
  bad.pop_max = EVO_POP_MAX + 2;
  CHECK(pgpe_workspace_bytes(&bad) == 0);
  bad = cfg;
  bad.P = 0;
  CHECK(pgpe_workspace_bytes(&bad) == 0);

  pgpe_state* st = NULL;
  CHECK(pgpe_create(&st, &cfg, NULL, NULL, NULL, NULL, NULL, NULL) == EVO_ERR_ARG);
  CHECK(strstr(evo_last_error(), "non-null") != NULL);
  CHECK(pgpe_create(NULL, &cfg, fake, fake, fake, fake, NULL, fake) == EVO_ERR_ARG);
  pgpe_config rule1 = cfg;
  rule1.sigma_rule = 1;
  CHECK(pgpe_create(&st, &rule1, fake, fake, fake, fake, NULL, fake) == EVO_ERR_ARG);
  pgpe_config clip = cfg;
  clip.optimizer = EVO_OPT_CLIPUP;
  clip.max_speed = 0.f;
  CHECK(pgpe_create(&st, &clip, fake, fake, fake, fake, NULL, fake) == EVO_ERR_ARG);
  CHECK(pgpe_create(&st, &cfg, fake, fake, fake, fake, NULL, fake) == EVO_OK && st != NULL);
  uint32_t t = 0;
  CHECK(pgpe_get_generation(st, &t) == EVO_OK && t == 1);
  CHECK(pgpe_set_generation(st, 0) == EVO_ERR_ARG);
  CHECK(pgpe_set_generation(st, 7) == EVO_OK && pgpe_get_generation(st, &t) == EVO_OK && t == 7);
  CHECK(pgpe_state_bytes(st) > 4 * 676 * 4);
  CHECK(pgpe_tell(st, (const float*)fake, NULL) == EVO_ERR_STATE);
  CHECK(pgpe_ask(st, 1, 63, fake, EVO_F32, NULL) == EVO_ERR_ARG);
  CHECK(pgpe_ask(st, 1, 66, fake, EVO_F32, NULL) == EVO_ERR_ARG);
  CHECK(pgpe_ask(st, 1, 64, fake, 7, NULL) == EVO_ERR_ARG);
  CHECK(pgpe_ask(st, 1, 64, (void*)0x1004, EVO_F32, NULL) == EVO_ERR_ARG);
  CHECK(pgpe_ask(st, 1, 64, NULL, EVO_F32, NULL) == EVO_ERR_ARG);
  CHECK(pgpe_tell_stored(st, (const float*)fake, NULL, NULL) != EVO_OK);
  CHECK(pgpe_state_export(st, NULL, 0, NULL) != EVO_OK);
  CHECK(pgpe_destroy(st) == EVO_OK);
  CHECK(pgpe_destroy(NULL) != EVO_OK || 1); /* either convention: must not crash */

  /* policy descriptions */
  policy_desc pd;
  memset(&pd, 0, sizeof pd);
  pd.kind = EVO_POLICY_MLP, pd.n_layers = 2, pd.dims[0] = 16, pd.dims[1] = 32, pd.dims[2] = 4;
  pd.act[0] = EVO_ACT_TANH, pd.act[1] = EVO_ACT_NONE, pd.dtype = EVO_F32;
  CHECK(policy_param_count(&pd) == 16 * 32 + 32 + 32 * 4 + 4);
  pd.dims[1] = 0;
  CHECK(policy_param_count(&pd) < 0);
  pd.dims[1] = 32, pd.n_layers = EVO_MAX_LAYERS + 1;
  CHECK(policy_param_count(&pd) < 0);
  pd.n_layers = 2, pd.act[0] = 9;
  CHECK(policy_param_count(&pd) < 0);
  CHECK(policy_param_count(NULL) < 0);
  policy_desc conv;
  memset(&conv, 0, sizeof conv);
  conv.kind = EVO_POLICY_CONVNET, conv.dims[0] = 28, conv.dims[1] = 8, conv.dims[2] = 16, conv.dims[3] = 10;
  CHECK(policy_param_count(&conv) == 9098);
  conv.dims[0] = 30;
  CHECK(policy_param_count(&conv) < 0);
  conv.dims[0] = 28, conv.dims[1] = 2000000000; /* sizes that would overflow 32-bit products are refused, not wrapped */
  CHECK(policy_param_count(&conv) < 0);
  policy_desc lstm;
  memset(&lstm, 0, sizeof lstm);
  lstm.kind = EVO_POLICY_LSTM_SEQ2SEQ, lstm.dims[0] = 13, lstm.dims[1] = 128, lstm.dims[2] = 10;
  CHECK(policy_param_count(&lstm) == 2 * (13 * 512 + 128 * 512 + 512) + 128 * 10 + 10);
  lstm.dims[0] = 0;
  CHECK(policy_param_count(&lstm) < 0);
  pd.act[0] = EVO_ACT_TANH;
  pd.kind = 17;
  CHECK(policy_param_count(&pd) < 0);
  pd.kind = EVO_POLICY_MLP;

  /* task descriptions and size queries */
  task_desc td;
  memset(&td, 0, sizeof td);
  td.kind = EVO_TASK_CLASSIFY, td.B = 512;
  CHECK(rollout_workspace_bytes(&td, &pd, 64) >= 64 * 8 * 4);
  CHECK(rollout_workspace_bytes(&td, &pd, 63) == 0 || rollout_workspace_bytes(&td, &pd, 63) > 0); /* no crash */
  CHECK(rollout_workspace_bytes(NULL, &pd, 64) == 0);
  td.kind = EVO_TASK_SPHERE, td.P = 8;
  CHECK(rollout_workspace_bytes(&td, NULL, 4) >= 16);
  td.kind = EVO_TASK_CARTPOLE;
  CHECK(rollout_workspace_bytes(&td, &pd, 4) == 0);
  td.kind = 99;
  CHECK(rollout_workspace_bytes(&td, &pd, 4) == 0);

  /* argument checks of the launching calls: all refused before any launch */
  td.kind = EVO_TASK_CLASSIFY, td.B = 512;
  CHECK(rollout(NULL, &pd, fake, 64, 1, (float*)fake, NULL) == EVO_ERR_ARG);
  CHECK(rollout(&td, &pd, NULL, 64, 1, (float*)fake, NULL) == EVO_ERR_ARG);
  CHECK(rollout(&td, &pd, fake, 0, 1, (float*)fake, NULL) == EVO_ERR_ARG);
  CHECK(rollout(&td, &pd, fake, 64, 1, (float*)fake, NULL) != EVO_OK); /* no observations, no workspace */
  CHECK(pop_forward(NULL, fake, (const float*)fake, 0, (float*)fake, 64, 8, NULL) == EVO_ERR_ARG);
  CHECK(pop_forward(&pd, NULL, (const float*)fake, 0, (float*)fake, 64, 8, NULL) == EVO_ERR_ARG);
  CHECK(pop_forward(&pd, fake, (const float*)fake, 0, (float*)fake, 0, 8, NULL) == EVO_ERR_ARG);
  CHECK(rollout_static_scratch(NULL, &pd, fake, 64, 1, (float*)fake, NULL) == EVO_ERR_ARG);
  CHECK(evo_centered_rank(NULL, 64, NULL, NULL, NULL) == EVO_ERR_ARG);
  CHECK(evo_centered_rank((const float*)fake, EVO_POP_MAX + 1, (uint32_t*)fake, (float*)fake, NULL) == EVO_ERR_ARG);
  CHECK(evo_philox_u32(1, 1, 0, 0, 0, 9, NULL, NULL) != EVO_OK);
  CHECK(evo_probe_rate(99, 1, NULL, (float*)fake, NULL) != EVO_OK);

  if (failures) {
    fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  printf("host checks passed\n");
  return 0;
}
