/* A plain C99 consumer of include/novak.h: proves the header is valid C, prints the layout of every
 * struct (so the Python mirror can be checked against what a C compiler really lays out) and calls the
 * entry points that need no GPU.  Built and run by tests/test_c_abi_from_c.py. */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "novak.h"

#define FIELD(type, name) printf("offset %s.%s %zu\n", #type, #name, offsetof(type, name))

int main(void) {
  novak_hparams hp, eff;
  novak_step_scalars sc;
  novak_chunk table[8];
  uint32_t warn = 77;
  int64_t numels[3] = {5, 0, 10000};
  int64_t needed = -1;
  int rc, i;

  printf("sizeof novak_hparams %zu\n", sizeof(novak_hparams));
  printf("sizeof novak_tensor_desc %zu\n", sizeof(novak_tensor_desc));
  printf("sizeof novak_step_scalars %zu\n", sizeof(novak_step_scalars));
  printf("sizeof novak_chunk %zu\n", sizeof(novak_chunk));
  printf("sizeof novak_info %zu\n", sizeof(novak_info));
  FIELD(novak_hparams, lr); FIELD(novak_hparams, la_k); FIELD(novak_hparams, auto_sync); FIELD(novak_hparams, layer_adaptation);
  FIELD(novak_hparams, auto_lr_gamma); FIELD(novak_hparams, clip_threshold); FIELD(novak_hparams, use_gc);
  FIELD(novak_hparams, beta_tau1); FIELD(novak_hparams, n_taylor); FIELD(novak_hparams, moment_dtype);
  FIELD(novak_tensor_desc, la_buf); FIELD(novak_tensor_desc, numel); FIELD(novak_tensor_desc, rows);
  FIELD(novak_step_scalars, decay); FIELD(novak_step_scalars, rectified_now); FIELD(novak_step_scalars, beta1_t);
  FIELD(novak_step_scalars, nesterov_mode);
  FIELD(novak_chunk, tensor); FIELD(novak_chunk, len);
  FIELD(novak_info, warnings); FIELD(novak_info, n_chunks); FIELD(novak_info, last_step); FIELD(novak_info, sync_due);
  FIELD(novak_info, n_centralized); FIELD(novak_info, moment_dtype);

  memset(&hp, 0, sizeof hp);
  hp.struct_size = sizeof hp;
  hp.lr = 1e-3; hp.beta1 = 0.9; hp.beta2 = 0.999; hp.eps = 1e-8; hp.weight_decay = 1e-2; hp.beta_n = 0.9;
  hp.la_alpha = 0.5; hp.la_k = 5; hp.rectified = 1; hp.decoupled_decay = 1;
  hp.nesterov_mode = NOVAK_NESTEROV_TRUE; hp.lookahead_mode = NOVAK_LOOKAHEAD_BASIC;
  hp.unrect_fallback = NOVAK_UNRECT_ADAM_DENOM; hp.mode = NOVAK_MODE_FAST;
  hp.auto_lr_gamma = 0.1; hp.trust_clip_lo = 0.1; hp.trust_clip_hi = 10.0; hp.auto_clip_lo = 0.1; hp.auto_clip_hi = 2.0;
  hp.beta_tau1 = 1000.0; hp.beta_tau2 = 5000.0;
  rc = novak_validate_hparams(&hp, &eff, &warn);
  printf("validate rc %d nesterov %d lookahead %d warn %u\n", rc, (int)eff.nesterov_mode, (int)eff.lookahead_mode, (unsigned)warn);
  hp.lr = -1.0;
  printf("validate_bad rc %d\n", novak_validate_hparams(&hp, &eff, &warn));
  hp.lr = 1e-3;
  rc = novak_compute_step_scalars(&eff, 6, &sc);
  printf("scalars rc %d rho_t %.17g r_t %.17g rectified_now %d step_size %.17g\n", rc, sc.rho_t, sc.r_t, (int)sc.rectified_now, sc.step_size);
  rc = novak_plan_chunks(numels, 3, 4096, NULL, 0, &needed);
  printf("plan rc %d needed %lld\n", rc, (long long)needed);
  rc = novak_plan_chunks(numels, 3, 4096, table, 8, &needed);
  for (i = 0; i < (int)needed; ++i) printf("chunk %d tensor %d offset %lld len %d\n", i, (int)table[i].tensor, (long long)table[i].offset, (int)table[i].len);
  printf("bytes %.1f %.1f\n", novak_bytes_per_param_step(NOVAK_LOOKAHEAD_NONE, NOVAK_GRAD_F32, 5, 1, 0),
         novak_bytes_per_param_step(NOVAK_LOOKAHEAD_MEMORY_EFFICIENT, NOVAK_GRAD_BF16, 5, 2, 1));
  {
    int64_t offs[3], role_elems = -1, stride = -1;
    rc = novak_plan_arena(numels, 3, offs, &role_elems, &stride);
    printf("arena rc %d offsets %lld %lld %lld role_elems %lld stride %lld\n", rc, (long long)offs[0], (long long)offs[1],
           (long long)offs[2], (long long)role_elems, (long long)stride);
  }
  printf("status %s\n", novak_status_string(NOVAK_ERR_MISALIGNED));
  {
    novak_handle *h = (novak_handle *)&hp;   /* must come back NULL */
    rc = novak_create(&h, &hp, NULL, 0, -1);
    printf("create_bad rc %d handle_null %d msg %s\n", rc, h == NULL, novak_last_error(NULL));
  }
  printf("destroy_null %d\n", novak_destroy(NULL));
  return 0;
}
