// Host-only part of the NOVAK update-step library: hyper-parameter validation and fast-path
// downgrade (paper sections 5.8 and 7.3), the per-step scalar prologue (Eq. 5-9, 18, 24a), the
// multi-tensor chunk planner and the algorithmic byte accounting (section 5.5).  No HIP calls here,
// so these entry points work on machines without a GPU.
#include "novak_internal.h"
#include "novak_prologue.h"

#include <cmath>
#include <cstdint>
#include <cstring>

namespace {

bool finite_all(const novak_hparams &hp) {
  const double vals[] = {hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.beta_n, hp.la_alpha,
                         hp.auto_lr_gamma, hp.trust_clip_lo, hp.trust_clip_hi, hp.auto_clip_lo, hp.auto_clip_hi,
                         hp.clip_threshold, hp.sparse_threshold, hp.beta_tau1, hp.beta_tau2};
  for (double x : vals)
    if (!std::isfinite(x)) return false;
  return true;
}

}  // namespace

extern "C" {

const char *novak_status_string(int status) {
  switch (status) {
    case NOVAK_OK: return "ok";
    case NOVAK_ERR_INVALID_ARG: return "invalid argument";
    case NOVAK_ERR_NULL_POINTER: return "null pointer";
    case NOVAK_ERR_MISALIGNED: return "misaligned pointer";
    case NOVAK_ERR_BAD_STEP: return "bad step number";
    case NOVAK_ERR_STATE: return "call not legal in the handle's current state";
    case NOVAK_ERR_HIP: return "HIP runtime error";
    case NOVAK_ERR_NOT_IMPLEMENTED: return "not implemented";
    case NOVAK_ERR_NO_MEMORY: return "out of memory";
    default: return "unknown status";
  }
}

int novak_validate_hparams(const novak_hparams *hp, novak_hparams *effective, uint32_t *warnings) {
  if (warnings) *warnings = 0;
  if (!hp) return NOVAK_ERR_NULL_POINTER;
  if (hp->struct_size != sizeof(novak_hparams)) return NOVAK_ERR_INVALID_ARG;
  if (!finite_all(*hp)) return NOVAK_ERR_INVALID_ARG;
  // section 5.8, "Hyperparameter validation"
  if (!(hp->lr > 0.0)) return NOVAK_ERR_INVALID_ARG;
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0)) return NOVAK_ERR_INVALID_ARG;
  if (!(hp->beta2 >= 0.0 && hp->beta2 < 1.0)) return NOVAK_ERR_INVALID_ARG;
  if (!(hp->weight_decay >= 0.0)) return NOVAK_ERR_INVALID_ARG;
  if (!(hp->beta_n >= 0.0 && hp->beta_n < 1.0)) return NOVAK_ERR_INVALID_ARG;
  if (!(hp->eps > 0.0)) return NOVAK_ERR_INVALID_ARG;
  if (hp->la_k < 1) return NOVAK_ERR_INVALID_ARG;
  // rho_inf = 2/(1-beta2) - 1 must be well defined when rectifying
  if (hp->rectified && !(hp->beta2 < 1.0 - 1e-8)) return NOVAK_ERR_INVALID_ARG;
  if (hp->nesterov_mode < NOVAK_NESTEROV_NONE || hp->nesterov_mode > NOVAK_NESTEROV_TRUE) return NOVAK_ERR_INVALID_ARG;
  if (hp->lookahead_mode < NOVAK_LOOKAHEAD_NONE || hp->lookahead_mode > NOVAK_LOOKAHEAD_BASIC) return NOVAK_ERR_INVALID_ARG;
  if (hp->unrect_fallback != NOVAK_UNRECT_ADAM_DENOM && hp->unrect_fallback != NOVAK_UNRECT_SGDM) return NOVAK_ERR_INVALID_ARG;
  if (hp->mode != NOVAK_MODE_FAST && hp->mode != NOVAK_MODE_RESEARCH) return NOVAK_ERR_INVALID_ARG;
  if (hp->lookahead_mode != NOVAK_LOOKAHEAD_NONE && !(hp->la_alpha > 0.0 && hp->la_alpha <= 1.0)) return NOVAK_ERR_INVALID_ARG;

  if (!(hp->clip_threshold >= 0.0) || !(hp->sparse_threshold >= 0.0)) return NOVAK_ERR_INVALID_ARG;
  if (hp->adaptive_beta && !(hp->beta_tau1 > 0.0 && hp->beta_tau2 > 0.0)) return NOVAK_ERR_INVALID_ARG;
  if (hp->n_taylor < 0) return NOVAK_ERR_INVALID_ARG;
  if (hp->moment_dtype != NOVAK_MOMENT_F32 && hp->moment_dtype != NOVAK_MOMENT_BF16_M) return NOVAK_ERR_INVALID_ARG;
  if (hp->layer_adaptation && !(hp->trust_clip_lo > 0.0 && hp->trust_clip_lo <= hp->trust_clip_hi)) return NOVAK_ERR_INVALID_ARG;
  if (hp->auto_lr) {
    if (!(hp->auto_lr_gamma > 0.0 && hp->auto_lr_gamma <= 1.0)) return NOVAK_ERR_INVALID_ARG;
    if (!(hp->auto_clip_lo > 0.0 && hp->auto_clip_lo <= hp->auto_clip_hi)) return NOVAK_ERR_INVALID_ARG;
  }

  novak_hparams eff = *hp;
  uint32_t warn = 0;
  // section 7.3: the fast path substitutes cheap variants for expensive ones and warns
  if (eff.mode == NOVAK_MODE_FAST) {
    if (eff.nesterov_mode == NOVAK_NESTEROV_TRUE) {
      eff.nesterov_mode = NOVAK_NESTEROV_APPROX;
      warn |= NOVAK_WARN_TRUE_NESTEROV_DOWNGRADED;
    }
    if (eff.lookahead_mode == NOVAK_LOOKAHEAD_BASIC) {
      eff.lookahead_mode = NOVAK_LOOKAHEAD_MEMORY_EFFICIENT;
      warn |= NOVAK_WARN_LOOKAHEAD_DOWNGRADED;
    }
  }
  eff.layer_adaptation = eff.layer_adaptation ? 1 : 0;
  eff.auto_lr = eff.auto_lr ? 1 : 0;
  eff.use_gc = eff.use_gc ? 1 : 0;
  eff.adaptive_beta = eff.adaptive_beta ? 1 : 0;
  // section 7.1: layer adaptation and auto-LR exist only in full-features mode
  if (eff.mode == NOVAK_MODE_FAST) {
    if (eff.layer_adaptation) {
      eff.layer_adaptation = 0;
      warn |= NOVAK_WARN_LAYER_ADAPTATION_DISABLED;
    }
    if (eff.auto_lr) {
      eff.auto_lr = 0;
      warn |= NOVAK_WARN_AUTO_LR_DISABLED;
    }
    if (eff.use_gc) {
      eff.use_gc = 0;
      warn |= NOVAK_WARN_GC_DISABLED;
    }
  }
  eff.rectified = eff.rectified ? 1 : 0;
  eff.decoupled_decay = eff.decoupled_decay ? 1 : 0;
  eff.auto_sync = eff.auto_sync ? 1 : 0;
  eff.device_step = eff.device_step ? 1 : 0;
  if (effective) *effective = eff;
  if (warnings) *warnings = warn;
  return NOVAK_OK;
}

int novak_compute_step_scalars(const novak_hparams *hp, int64_t step, novak_step_scalars *out) {
  if (!hp || !out) return NOVAK_ERR_NULL_POINTER;
  if (hp->struct_size != sizeof(novak_hparams)) return NOVAK_ERR_INVALID_ARG;
  if (step < 1) return NOVAK_ERR_BAD_STEP;
  novak_step_scalars_impl(*hp, step, out);
  return NOVAK_OK;
}

int novak_plan_chunks(const int64_t *numels, int32_t n_tensors, int64_t chunk_elems, novak_chunk *out,
                      int64_t capacity, int64_t *n_chunks) {
  if (!n_chunks || (n_tensors > 0 && !numels)) return NOVAK_ERR_NULL_POINTER;
  if (n_tensors < 0 || capacity < 0 || (capacity > 0 && !out)) return NOVAK_ERR_INVALID_ARG;
  if (chunk_elems < NOVAK_CHUNK_MIN || chunk_elems > NOVAK_CHUNK_MAX || (chunk_elems & (chunk_elems - 1)) != 0)
    return NOVAK_ERR_INVALID_ARG;
  int64_t n = 0;
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t numel = numels[t];
    if (numel < 0) return NOVAK_ERR_INVALID_ARG;
    for (int64_t off = 0; off < numel; off += chunk_elems) {
      if (n < capacity) {
        const int64_t rest = numel - off;
        out[n].offset = off;
        out[n].tensor = t;
        out[n].len = static_cast<int32_t>(rest < chunk_elems ? rest : chunk_elems);
      }
      ++n;
    }
  }
  *n_chunks = n;
  return NOVAK_OK;
}

int novak_plan_arena(const int64_t *numels, int32_t n_tensors, int64_t *tensor_offsets, int64_t *role_elems,
                     int64_t *role_stride_bytes) {
  if (n_tensors < 0) return NOVAK_ERR_INVALID_ARG;
  if ((n_tensors > 0 && !numels) || !role_elems || !role_stride_bytes) return NOVAK_ERR_NULL_POINTER;
  const int64_t limit = INT64_MAX / 8;
  int64_t off = 0;
  for (int32_t i = 0; i < n_tensors; ++i) {
    if (numels[i] < 0 || numels[i] > limit - off) return NOVAK_ERR_INVALID_ARG;
    if (tensor_offsets) tensor_offsets[i] = off;
    off += (numels[i] + NOVAK_ARENA_TENSOR_ALIGN - 1) / NOVAK_ARENA_TENSOR_ALIGN * NOVAK_ARENA_TENSOR_ALIGN;
  }
  *role_elems = off;
  const int64_t bytes = off * 4;    // the widest role holds 4-byte elements
  *role_stride_bytes = (bytes + NOVAK_ARENA_ROLE_PERIOD - 1) / NOVAK_ARENA_ROLE_PERIOD * NOVAK_ARENA_ROLE_PERIOD + NOVAK_ARENA_ROLE_SKEW;
  return NOVAK_OK;
}

double novak_bytes_per_param_step(int32_t lookahead_mode, int32_t grad_dtype, int32_t la_k, int32_t window_pos,
                                  int32_t fused_sync) {
  // section 5.5: theta, g, m, v read; theta, m, v written
  double bytes = 3 * 4 + (grad_dtype == NOVAK_GRAD_BF16 ? 2 : 4) + 3 * 4;
  if (lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT) {
    const bool first = window_pos == 1, last = window_pos == la_k;
    if (!first) bytes += 4;                      // buffer read (the first step of a window overwrites it)
    if (!(last && fused_sync && la_k > 1)) bytes += 4;  // buffer written (skipped when the sync is fused)
  } else if (lookahead_mode == NOVAK_LOOKAHEAD_BASIC) {
    if (window_pos == la_k && fused_sync) bytes += 8;   // slow weights read and written
  }
  return bytes;
}

double novak_bytes_per_param_scaled_step(int32_t lookahead_mode, int32_t grad_dtype, int32_t la_k, int32_t window_pos,
                                         int32_t fused_sync) {
  // the single-pass figure plus pass 2 reading theta, m, v again
  return novak_bytes_per_param_step(lookahead_mode, grad_dtype, la_k, window_pos, fused_sync) + 12;
}

double novak_bytes_per_param_moment_saving(int32_t moment_dtype, int32_t two_pass) {
  if (moment_dtype != NOVAK_MOMENT_BF16_M) return 0;
  return two_pass ? 6 : 4;
}

double novak_bytes_per_param_clip(int32_t grad_dtype) { return grad_dtype == NOVAK_GRAD_BF16 ? 2 : 4; }

double novak_bytes_per_param_sync(int32_t lookahead_mode) {
  if (lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT) return 8;   // buffer read, theta written
  if (lookahead_mode == NOVAK_LOOKAHEAD_BASIC) return 16;             // theta, slow read; both written
  return 0;
}

}  // extern "C"
