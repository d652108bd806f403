// The per-step scalar prologue (Phases 3, 5, 6 and the constants of Phases 8-10) as one function that compiles
// for the host AND for the device: novak_compute_step_scalars / novak_step evaluate it on the host, the
// device-step mode (step count in device memory, for callers that replay a captured HIP graph) evaluates it in a
// prologue kernel (one lane per step).  Double arithmetic in both places; 1 - beta^t through expm1(t log beta) (section 5.8).
#ifndef NOVAK_PROLOGUE_H_
#define NOVAK_PROLOGUE_H_

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "novak_internal.h"

__host__ __device__ inline double novak_one_minus_pow(double beta, int64_t t) {
  if (beta == 0.0) return 1.0;
  return -expm1(static_cast<double>(t) * log(beta));
}

// Scalars of step `step` (>= 1) for validated hyper-parameters (Eq. 3-9, 18, 24a).
__host__ __device__ inline void novak_step_scalars_impl(const novak_hparams &hp, int64_t step, novak_step_scalars *out) {
  novak_step_scalars s = novak_step_scalars();
  s.bc1 = novak_one_minus_pow(hp.beta1, step);
  s.bc2 = novak_one_minus_pow(hp.beta2, step);
  s.rho_inf = 2.0 / (1.0 - hp.beta2) - 1.0;                         // Eq. 6
  const double beta2_pow_t = 1.0 - s.bc2;
  s.rho_t = s.rho_inf - 2.0 * static_cast<double>(step) * beta2_pow_t / s.bc2;  // Eq. 7
  s.r_t = 1.0;
  s.rectified_now = 0;
  s.denom_on = 1;
  if (hp.rectified) {
    if (s.rho_t >= 5.0) {                                            // Eq. 8, rectified branch
      s.rectified_now = 1;
      const double num = (s.rho_t - 4.0) * (s.rho_t - 2.0) * s.rho_inf;
      const double den = (s.rho_inf - 4.0) * (s.rho_inf - 2.0) * s.rho_t;
      s.r_t = sqrt(num / den);                                       // Eq. 9
    } else if (hp.unrect_fallback == NOVAK_UNRECT_SGDM) {
      s.denom_on = 0;
    }
  }
  s.beta1_t = hp.beta1;
  s.beta2_t = hp.beta2;
  if (hp.adaptive_beta) {                                            // Eq. 3-4
    s.beta1_t = hp.beta1 * (1.0 - exp(-static_cast<double>(step) / hp.beta_tau1));
    s.beta2_t = hp.beta2 * (1.0 - exp(-static_cast<double>(step) / hp.beta_tau2));
  }
  s.nesterov_mode = hp.nesterov_mode;                                // automatic fallback of the true variant
  if (hp.nesterov_mode == NOVAK_NESTEROV_TRUE && hp.n_taylor > 0 && step > hp.n_taylor) s.nesterov_mode = NOVAK_NESTEROV_APPROX;
  s.step_size = hp.lr * s.r_t;                                       // Eq. 24a
  s.decay = hp.decoupled_decay ? 1.0 - hp.lr * hp.weight_decay : 1.0;  // Eq. 18
  *out = s;
}

#endif  // NOVAK_PROLOGUE_H_
