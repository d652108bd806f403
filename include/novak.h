/*
 * novak.h - C ABI of the MI355X (gfx950) implementation of the NOVAK optimizer's fused update step.
 *
 * What the library computes, per parameter element and per step t (t = 1 on the first step), in
 * the paper's notation (section 4; phase order of section 5.1 / Table 2):
 *
 *   g~  = g + beta_n (g - m_{t-1})                         Nesterov approximation       (Eq. 13)
 *   m_t = beta1 m_{t-1} + (1-beta1) g~                     first moment                 (Eq. 1)
 *   v_t = beta2 v_{t-1} + (1-beta2) g~^2                   second moment                (Eq. 2)
 *   m^  = m_t / (1-beta1^t),  v^ = v_t / (1-beta2^t)       bias correction              (Eq. 5)
 *   u   = m^ / (sqrt(v^) + eps)                            update direction             (Eq. 17)
 *   u   = beta1 m^ + (1-beta1) u                           classical Nesterov blend     (Eq. 16)
 *   theta_t = theta_{t-1} (1 - alpha lambda) - alpha r_t u decoupled decay, then update (Eq. 18, 24, 24a)
 *
 * with the rectification schedule rho_inf, rho_t, r_t of Eq. 6-9 computed once per step on the
 * host in double precision, and the lookahead slow-weight synchronisation of section 4.7 every
 * la_k steps (Eq. 28-31; the averaging form stated in the proof of Theorem 6.2).
 *
 * All tensor memory is DEVICE memory owned by the caller (fp32, contiguous).  The library owns only
 * the handle, its chunk table and a small gradient-pointer table.  Every call returns a status
 * code; nothing throws or aborts across this boundary.
 *
 * Ordering.  Every call returns as soon as its kernels are enqueued on the HIP stream the caller passes;
 * nothing synchronises.  All calls on one handle must therefore be STREAM-ORDERED, not merely
 * non-overlapping on the host: the handle's device tables (gradient-pointer list, reduction buffers, row
 * means, clipping factor) are single-buffered and protected only by the order of the stream they were
 * last used on.  Use one stream per handle, or make the next call's stream wait (hipStreamWaitEvent) on
 * an event recorded after the previous call.  Two host threads must not call into one handle at once.
 */
#ifndef NOVAK_H_
#define NOVAK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct novak_handle novak_handle;

/* ---- status codes ------------------------------------------------------------------------- */
enum {
  NOVAK_OK = 0,
  NOVAK_ERR_INVALID_ARG = 1,      /* a hyper-parameter breaks a rule of section 5.8 / 7.3, or a bad size */
  NOVAK_ERR_NULL_POINTER = 2,     /* a required pointer is NULL */
  NOVAK_ERR_MISALIGNED = 3,       /* a tensor pointer is not aligned to its element size */
  NOVAK_ERR_BAD_STEP = 4,         /* step < 1, or not last step + 1 on this handle */
  NOVAK_ERR_STATE = 5,            /* call not legal now (sync not due / sync pending / no lookahead) */
  NOVAK_ERR_HIP = 6,              /* a HIP runtime call failed; see novak_last_error() */
  NOVAK_ERR_NOT_IMPLEMENTED = 7,  /* the entry point does not cover a requested feature (novak_step_static: layer adaptation, auto-LR, centralization) */
  NOVAK_ERR_NO_MEMORY = 8
};

/* ---- enumerations of Algorithm 1's header (section 5.2) -------------------------------------- */
enum { NOVAK_NESTEROV_NONE = 0, NOVAK_NESTEROV_APPROX = 1, NOVAK_NESTEROV_CLASSICAL = 2, NOVAK_NESTEROV_TRUE = 3 };
enum { NOVAK_LOOKAHEAD_NONE = 0, NOVAK_LOOKAHEAD_MEMORY_EFFICIENT = 1, NOVAK_LOOKAHEAD_BASIC = 2 };
/* What a step is while rho_t < 5 (Eq. 8 is silent about the denominator):
 * ADAM_DENOM keeps u = m^/(sqrt(v^)+eps) with r_t = 1; SGDM uses u = m^ (original RAdam). */
enum { NOVAK_UNRECT_ADAM_DENOM = 0, NOVAK_UNRECT_SGDM = 1 };
/* Dual-mode control of section 7.1: FAST is the paper's fast path, RESEARCH its full-features mode. */
enum { NOVAK_MODE_FAST = 0, NOVAK_MODE_RESEARCH = 1 };
enum { NOVAK_GRAD_F32 = 0, NOVAK_GRAD_BF16 = 1 };
/* Storage of the first moment.  BF16_M (the paper's "multi-precision" outlook, not part of its method):
 * exp_avg is an array of bfloat16, rounded to nearest-even once per step from the fp32 value of Eq. 1;
 * the rounded value is the m_t the rest of the step uses.  exp_avg_sq stays fp32 (with beta2 = 0.999 its
 * per-step change is below half a bfloat16 ulp and a rounded v would stop moving). */
enum { NOVAK_MOMENT_F32 = 0, NOVAK_MOMENT_BF16_M = 1 };

/* warning bits reported by novak_validate_hparams / novak_get_info (section 7.3: downgrades warn) */
enum {
  NOVAK_WARN_TRUE_NESTEROV_DOWNGRADED = 1u << 0,  /* FAST + TRUE        -> APPROX           */
  NOVAK_WARN_LOOKAHEAD_DOWNGRADED = 1u << 1,      /* FAST + BASIC       -> MEMORY_EFFICIENT */
  NOVAK_WARN_LAYER_ADAPTATION_DISABLED = 1u << 2, /* FAST + layer_adaptation -> off (section 7.1) */
  NOVAK_WARN_AUTO_LR_DISABLED = 1u << 3,          /* FAST + auto_lr          -> off (section 7.1) */
  NOVAK_WARN_GC_DISABLED = 1u << 4                /* FAST + use_gc           -> off (section 7.1) */
};

/* ---- hyper-parameters (host memory, plain data) -------------------------------------------------
 * Rules checked (section 5.8 "Hyperparameter validation", section 7.3): lr > 0; beta1, beta2 in
 * [0,1); weight_decay >= 0; beta_n in [0,1); la_k >= 1; eps > 0; beta2 < 1 - 1e-8 when rectified;
 * la_alpha in (0,1] when lookahead is on (the paper's open bound at 1 is relaxed so that the
 * alpha_LA = 1 fixed point can be exercised); auto_lr_gamma in (0,1] and 0 < lo <= hi for both clip
 * ranges when the respective scaling is on; clip_threshold >= 0; sparse_threshold >= 0.  All values
 * must be finite. */
typedef struct novak_hparams {
  size_t struct_size;      /* sizeof(novak_hparams); guards against layout mismatch */
  double lr;               /* alpha   */
  double beta1, beta2;     /* moment decay rates */
  double eps;              /* epsilon, added outside the root (Eq. 17) */
  double weight_decay;     /* lambda  */
  double beta_n;           /* Nesterov coefficient of Eq. 13 (no default in the paper) */
  double la_alpha;         /* alpha_LA */
  int32_t la_k;            /* k: steps per lookahead window */
  int32_t rectified;       /* 0/1: RAdam rectification (Eq. 6-9) */
  int32_t decoupled_decay; /* 1: Eq. 18; 0: classic L2, g <- g + lambda*theta (a reading; paper gives no formula) */
  int32_t nesterov_mode;   /* NOVAK_NESTEROV_*; TRUE means `grads` were evaluated at theta + beta_n m (Eq. 10-11) by the caller */
  int32_t lookahead_mode;  /* NOVAK_LOOKAHEAD_* */
  int32_t unrect_fallback; /* NOVAK_UNRECT_* */
  int32_t mode;            /* NOVAK_MODE_* */
  int32_t auto_sync;       /* 1: novak_step performs the sync itself, fused into the k-th step's pass */
  /* Full-features scalings of alpha_eff = alpha * r_t * lambda_trust * alpha_auto (Eq. 24a); RESEARCH mode only.
   * The trust ratio turns the step into two passes over the state (per-tensor norms of the direction first, then the
   * update).  Auto-LR alone needs global norms of inputs only: one extra read of the gradients and of the parameters,
   * then the single-pass step. */
  int32_t layer_adaptation; /* 1: per-tensor trust ratio ||theta||/||u||, u of Eq. 17, clipped (Eq. 19, 25); 1 when a norm is 0 */
  int32_t auto_lr;          /* 1: alpha_auto = clip(g_bar/theta_bar) from EMAs of the global gradient and parameter
                               norms (Eq. 20-22); needs novak_set_auto_lr_state */
  double auto_lr_gamma;     /* gamma of Eq. 20-21, in (0,1]; the paper uses 0.1 */
  double trust_clip_lo, trust_clip_hi;   /* clip range of Eq. 19; the paper uses [0.1, 10]; 0 < lo <= hi */
  double auto_clip_lo, auto_clip_hi;     /* clip range of Eq. 22; the paper uses [0.1, 2];  0 < lo <= hi */
  /* Phase 2 / Phase 8 options, legal in both modes. */
  double clip_threshold;    /* c_clip >= 0 on the GLOBAL gradient norm (sections 5.8, 7.3), applied before any other
                               processing; 0 = off.  Costs one extra read of the gradients per step. */
  double sparse_threshold;  /* tau >= 0 of Eq. 27: the base direction u is zeroed where |u| <= tau; 0 = off */
  int32_t use_gc;           /* 1: gradient centralization (Eq. 26) on tensors whose descriptor gives rows >= 1; RESEARCH
                               mode only; runs after clipping, before the Nesterov approximation; costs one extra
                               read of those tensors' gradients per step */
  int32_t adaptive_beta;    /* 1: beta_i(t) = beta_i (1 - exp(-t/tau_i)) in the moment updates (Eq. 3-4); bias correction,
                               rectification and the classical blend keep the base betas, as printed */
  double beta_tau1, beta_tau2; /* tau_1, tau_2 of Eq. 3-4 (> 0 when adaptive_beta); the paper uses 1000 and 5000 */
  int64_t n_taylor;         /* TRUE Nesterov behaves as APPROX for steps t > n_taylor (sections 4.4, 5.8: 100-200);
                               0 = never; ignored for the other modes */
  int32_t moment_dtype;     /* NOVAK_MOMENT_*: element type of every tensor's exp_avg array */
  int32_t device_step;      /* 1: the step count t lives in DEVICE memory (novak_set_step_counter) and the scalar prologue runs
                               in a small kernel on the device, so that a novak_step captured into a HIP graph
                               advances by itself on every replay; novak_step's `step` argument must then be 0.  Every
                               option of the step is available; lookahead needs auto_sync = 1 (nobody on the host knows
                               when a sync is due). */
} novak_hparams;

/* One parameter tensor.  All pointers are DEVICE pointers to contiguous fp32 arrays of `numel`
 * elements, 4-byte aligned (16-byte alignment of every pointer selects the 128-bit path; any other
 * alignment is handled element-wise).  They must stay valid and fixed until novak_destroy, and no
 * two arrays may overlap.  numel == 0 is allowed.
 *   la_buf: the single lookahead buffer; required unless lookahead is NONE.  With auto_sync its
 *     contents are unspecified between a fused sync and the next step (which overwrites it).
 *     MEMORY_EFFICIENT: running blend (1-alpha_LA)*slow_0 + (alpha_LA/k)*sum of the window's iterates,
 *       which equals Eq. 30's right-hand side when the window is full (one buffer instead of the
 *       Delta + theta_0^slow pair of Table 3).
 *     BASIC: the slow weights theta^slow. */
typedef struct novak_tensor_desc {
  void *param;       /* theta, updated in place   */
  void *exp_avg;     /* m, updated in place (fp32; bfloat16, 2-byte aligned, with NOVAK_MOMENT_BF16_M) */
  void *exp_avg_sq;  /* v, updated in place       */
  void *la_buf;      /* see above; may be NULL when lookahead is NONE */
  int64_t numel;
  int64_t rows;      /* Eq. 26: size of the first dimension if the tensor has more than one dimension, else 0
                        (not centralized); must divide numel.  Ignored unless use_gc is on. */
} novak_tensor_desc;

/* Per-step scalars (Phases 5-6), as the host prologue computes them in double. */
typedef struct novak_step_scalars {
  double bc1, bc2;         /* 1-beta1^t, 1-beta2^t via -expm1(t log beta) (section 5.8) */
  double rho_inf, rho_t;   /* Eq. 6, 7 */
  double r_t;              /* Eq. 9, or 1 when rectification is off or rho_t < 5 */
  double step_size;        /* alpha * r_t (Eq. 24a with lambda_trust = alpha_auto = 1) */
  double decay;            /* 1 - alpha*lambda (Eq. 18), or 1 with coupled decay */
  int32_t rectified_now;   /* rectified && rho_t >= 5 */
  int32_t denom_on;        /* 0 only in the SGDM fallback while rho_t < 5 */
  double beta1_t, beta2_t; /* betas used by the moment updates at this step (Eq. 3-4, or the base values) */
  int32_t nesterov_mode;   /* variant in force at this step (TRUE -> APPROX after n_taylor steps) */
  int32_t reserved0;
} novak_step_scalars;

/* One entry of the multi-tensor chunk table: `len` elements of tensor `tensor` starting at `offset`. */
typedef struct novak_chunk {
  int64_t offset;
  int32_t tensor;
  int32_t len;
} novak_chunk;

typedef struct novak_info {
  size_t struct_size;
  int32_t nesterov_mode;     /* effective, after the fast-path downgrade */
  int32_t lookahead_mode;    /* effective */
  uint32_t warnings;         /* NOVAK_WARN_* */
  int32_t n_tensors;
  int64_t n_chunks;
  int64_t chunk_elems;
  int64_t total_numel;
  int64_t last_step;         /* 0 before the first step on this handle */
  int32_t sync_due;          /* 1 between a k-th step and its novak_lookahead_sync (auto_sync off) */
  int32_t device_id;
  int32_t layer_adaptation;  /* effective */
  int32_t auto_lr;           /* effective */
  int32_t use_gc;            /* effective */
  int32_t n_centralized;     /* tensors that are centralized (use_gc on and rows >= 1) */
  int32_t moment_dtype;      /* NOVAK_MOMENT_* */
  int32_t reserved0;
} novak_info;

/* tuning keys for novak_set_tuning */
enum {
  NOVAK_TUNE_CHUNK_ELEMS = 0,   /* elements per chunk-table entry; a power of two in [4096, 2^24] (default 16384; a handle that
                                   runs a gradient pre-pass starts with 65536, 16384 or 4096 by the size of its list) */
  NOVAK_TUNE_NONTEMPORAL = 1,   /* 0/1: non-temporal hints on the streaming loads and stores */
  NOVAK_TUNE_VEC_PER_LANE = 2,  /* 1, 2 or 4: 128-bit accesses per stream per lane */
  NOVAK_TUNE_THREADS = 3,       /* 64, 128 or 256 threads per workgroup; a workgroup covers threads*4*vec_per_lane elements */
  NOVAK_TUNE_WAVES_PER_CU = 4,  /* 0..32: cap on waves resident per compute unit (bounds the bytes in flight);
                                   0 = chosen per kernel variant from its number of streams */
  NOVAK_TUNE_PREPASS_WAVES_PER_CU = 5  /* the same for the gradient pre-pass (clipping norm / row means), a read-only
                                   kernel whose waves hold 16 KB in flight each; 0 = chosen by gradient type */
};

/* ---- host-only helpers (no GPU needed) -------------------------------------------------------- */

/* Validates `hp` by the rules above and writes the effective hyper-parameters (after the fast-path
 * downgrades of section 7.3) to `effective` and the NOVAK_WARN_* bits to `warnings` (either may be
 * NULL).  Returns NOVAK_OK, NOVAK_ERR_NULL_POINTER or NOVAK_ERR_INVALID_ARG; RESEARCH-mode features
 * outside the update step are not representable in novak_hparams, so nothing maps to
 * NOT_IMPLEMENTED here. */
int novak_validate_hparams(const novak_hparams *hp, novak_hparams *effective, uint32_t *warnings);

/* Scalars of step `step` (>= 1) for validated hyper-parameters (Eq. 5-9, 18, 24a).  Host memory. */
int novak_compute_step_scalars(const novak_hparams *hp, int64_t step, novak_step_scalars *out);

/* Cuts tensors of `numels[i]` elements into chunks of at most `chunk_elems` elements (a power of two
 * in [4096, 2^24]), in tensor
 * order; a chunk never spans two tensors and empty tensors produce none.  Writes up to `capacity`
 * entries to `out` (may be NULL with capacity 0 to query) and the total count to `n_chunks`. */
int novak_plan_chunks(const int64_t *numels, int32_t n_tensors, int64_t chunk_elems,
                      novak_chunk *out, int64_t capacity, int64_t *n_chunks);

/* Recommended placement of the five per-parameter arrays ("roles": theta, exp_avg, exp_avg_sq, la_buf,
 * gradient) of a tensor list inside ONE device allocation; host arithmetic only, the caller allocates.
 * Tensor i of role r (element size e_r bytes) starts at byte  r * (*role_stride_bytes) + tensor_offsets[i] * e_r
 * of the allocation, which must hold (*role_stride_bytes) bytes per role used.  Tensors start at multiples
 * of NOVAK_ARENA_TENSOR_ALIGN elements inside a role, so that the 1 KB a wave reads of each array never
 * straddles a 1 KB boundary, and consecutive roles are NOVAK_ARENA_ROLE_SKEW bytes apart modulo
 * NOVAK_ARENA_ROLE_PERIOD.  The library accepts any placement (see novak_tensor_desc); this one measured
 * 1-2 % more bandwidth on MI355X than a spacing that is a multiple of the period, and 3-4 % more than
 * separately allocated arrays, whose relative placement is up to the driver (-10 % .. +1 % from run to run).  `tensor_offsets` (n_tensors entries, elements) may be NULL; `role_elems` receives the padded
 * element count of one role. */
#define NOVAK_ARENA_TENSOR_ALIGN 256
#define NOVAK_ARENA_ROLE_PERIOD 8192
#define NOVAK_ARENA_ROLE_SKEW 2048
int novak_plan_arena(const int64_t *numels, int32_t n_tensors, int64_t *tensor_offsets, int64_t *role_elems,
                     int64_t *role_stride_bytes);

/* Device memory for such an arena: `bytes` bytes on device `device_id`, requested as physically contiguous
 * memory first (hipExtMallocWithFlags with hipDeviceMallocContiguous) and, if the driver cannot provide
 * that, as an ordinary hipMalloc allocation.  `*contiguous` (may be NULL) says which one it is.  On MI355X
 * the step kernel measured 6.73 TB/s on a contiguous arena against 6.5-6.6 TB/s on an ordinary allocation
 * of the same layout (whose physical placement, and with it the bandwidth, varies with what ran on the
 * device before).  The contents are NOT initialised.  Release with novak_arena_free after the last kernel
 * that uses the memory has finished; the library never frees it by itself. */
int novak_arena_alloc(int32_t device_id, size_t bytes, void **ptr, int32_t *contiguous);
int novak_arena_free(int32_t device_id, void *ptr);

/* The same memory for a PyTorch caller, without giving up torch's own allocator interface: the two
 * functions below have the signatures torch.cuda.memory.CUDAPluggableAllocator expects, so that
 *     alloc = torch.cuda.memory.CUDAPluggableAllocator(PATH_TO_THIS_LIBRARY, "novak_torch_malloc", "novak_torch_free")
 *     pool = torch.cuda.MemPool(alloc.allocator())
 *     with torch.cuda.use_mem_pool(pool): ... create parameters, gradients and optimizer state ...
 * makes torch's caching allocator take the segments of that pool from here.  A request of 1 MiB or more is
 * served like novak_arena_alloc (physically contiguous when the driver can, ordinary otherwise) with the
 * returned address NOVAK_ARENA_ROLE_SKEW bytes further along, modulo NOVAK_ARENA_ROLE_PERIOD, than that of
 * the previous large request; smaller requests are plain hipMalloc.  On MI355X five arrays allocated this
 * way measured the same bandwidth as one planned arena (6.7-6.8 TB/s against 6.3-6.5 TB/s for torch's default
 * allocations).  `stream` is ignored; returns NULL when the device is out of memory.
 * novak_torch_alloc_stats reports how many allocations made here are alive and how many of those are
 * physically contiguous (either pointer may be NULL). */
void *novak_torch_malloc(ptrdiff_t size, int device, void *stream);
void novak_torch_free(void *ptr, ptrdiff_t size, int device, void *stream);
void novak_torch_alloc_stats(int64_t *live, int64_t *live_contiguous);

/* Algorithmic HBM bytes per parameter of one step (section 5.5: 4 streams read + 3 written, 4 B
 * each; gradients 2 B when bf16; plus the lookahead buffer traffic of that step).  `window_pos` is
 * the step's 1-based position in its lookahead window (ignored when lookahead is NONE);
 * `fused_sync` says whether the k-th step also performs the sync. */
double novak_bytes_per_param_step(int32_t lookahead_mode, int32_t grad_dtype, int32_t la_k,
                                  int32_t window_pos, int32_t fused_sync);
/* The same for a two-pass step (layer_adaptation or auto_lr on): pass 1 reads theta, g, m, v and writes
 * m, v; pass 2 reads theta, m, v and writes theta, plus the lookahead traffic; the per-wave norm
 * partials (16 bytes per 256 elements, written and read once) are not counted. */
double novak_bytes_per_param_scaled_step(int32_t lookahead_mode, int32_t grad_dtype, int32_t la_k,
                                         int32_t window_pos, int32_t fused_sync);
/* Bytes per parameter that NOVAK_MOMENT_BF16_M removes from a step: 4 single-pass (m read and written
 * at 2 bytes instead of 4), 6 two-pass (m is read twice). */
double novak_bytes_per_param_moment_saving(int32_t moment_dtype, int32_t two_pass);
/* Algorithmic bytes per parameter of the clipping pre-pass (one read of the gradients). */
double novak_bytes_per_param_clip(int32_t grad_dtype);
/* Algorithmic bytes per parameter of the separate sync kernel. */
double novak_bytes_per_param_sync(int32_t lookahead_mode);

const char *novak_status_string(int status);

/* ---- device entry points ---------------------------------------------------------------------- */

/* Algorithm 1's header (section 5.2: inputs, hyper-parameters, initialisation) as an object: validates
 * `hp` by the rules of section 5.8 and applies the fast-path downgrades of section 7.3, checks every
 * descriptor, builds the multi-tensor chunk table and uploads it to device `device_id`.  Allocates no
 * parameter-sized memory and launches no kernel (m_0 = v_0 = 0 and Eq. 28 are the caller's buffers and
 * novak_lookahead_init).  `tensors` is host memory and is copied.  n_tensors >= 0.  A list that one
 * kernel launch cannot cover (more than 2^32 - 1 threads, about 1.7e10 elements) is refused with
 * NOVAK_ERR_INVALID_ARG.  On failure *out is NULL and novak_last_error(NULL) holds the reason. */
int novak_create(novak_handle **out, const novak_hparams *hp, const novak_tensor_desc *tensors,
                 int32_t n_tensors, int32_t device_id);

/* Eq. 28: writes the initial lookahead state from the current theta (la_buf <- theta) for every
 * tensor.  Call once at the start of training; not when resuming with preserved buffers.
 * NOVAK_ERR_STATE when lookahead is NONE. */
int novak_lookahead_init(novak_handle *h, void *hip_stream);

/* One optimizer step (Phases 2-9 and the lookahead accumulation of Phase 10) for all tensors in one
 * kernel launch.  `grads` is a HOST array of n_tensors DEVICE pointers to the gradients (fp32, or
 * bf16 bit patterns when grad_dtype is NOVAK_GRAD_BF16), contiguous, numel elements each, aligned
 * to the element size.  `step` is t, 1-based; on a fresh handle any t >= 1 is accepted (resume),
 * afterwards it must be the previous step + 1.  With lookahead on and auto_sync off, the step with
 * t mod k == 0 leaves the handle in "sync due" state and the next call must be
 * novak_lookahead_sync; with auto_sync on, that step applies Eq. 30-31 itself.  In device-step mode `step` must be 0. */
int novak_step(novak_handle *h, void *const *grads, int32_t grad_dtype, int64_t step, void *hip_stream);

/* Auto-LR state (Table 3: two scalars): `ema` is a DEVICE pointer to two doubles owned by the caller,
 * g_bar then theta_bar (Eq. 20-21), zero before the first step; the library updates them every step.
 * Required before the first novak_step when auto_lr is on (else NOVAK_ERR_STATE there).  Keeping the
 * two values is what resuming needs. */
int novak_set_auto_lr_state(novak_handle *h, void *ema);

/* Device-step mode (hp.device_step = 1): `counter` is a DEVICE pointer to one int64 owned by the caller, 8-byte aligned: the
 * number of steps taken so far (0 before the first step; when resuming, the last t).  A step is number counter + 1: a small
 * prologue kernel reads the counter and evaluates Eq. 5-9 in double (rounded once to fp32 like the host prologue), and the
 * step's last kernel stores the new count.  Eagerly that prologue runs in front of every step.  Under stream capture the
 * first novak_step of a capture writes the records of the next 64 steps at once and the following captured steps use them in
 * turn, so a replayed graph reads the counter when it starts and is otherwise self-contained (one prologue per 64 steps).
 * Required before the first novak_step in that mode (else NOVAK_ERR_STATE there); NOVAK_ERR_STATE on a handle in host-step
 * mode.  Whoever changes the counter's value calls this function again.  To capture steps into a HIP graph: take one step
 * eagerly first (it uploads the gradient-pointer list, which a capture cannot), keep the gradient buffers and the list fixed,
 * then capture any number of novak_step calls on the capture stream (a call whose gradient-pointer list differs from the
 * previous call's is refused under capture with NOVAK_ERR_STATE); each replay takes that many more steps.  In this mode the
 * handle does not track t: novak_get_info reports last_step = 0, and the residency of the step kernel is chosen for the
 * lookahead phase with the most streams. */
int novak_set_step_counter(novak_handle *h, void *counter);

/* Monitoring: copies lambda_trust * alpha_auto of the last step (a factor that is off counts as 1), one float per tensor, to HOST
 * memory `out` (n_tensors floats).  Waits for `hip_stream` first.  NOVAK_ERR_STATE on a handle with neither scaling. */
int novak_copy_tensor_scales(novak_handle *h, float *out, void *hip_stream);

/* True Nesterov, Eq. 10: writes the extrapolated parameters theta + beta_n * m of every tensor to the
 * caller's buffers (`out` is a HOST array of n_tensors DEVICE pointers to fp32 arrays of numel elements,
 * 4-byte aligned, not overlapping the state).  The caller evaluates the gradient there (Eq. 11) and
 * passes it to novak_step; theta itself is left untouched, so there is nothing to restore.  One launch;
 * 12 bytes per parameter (10 with a bfloat16 m).  Legal in any Nesterov mode.  The list is copied before the
 * call returns. */
int novak_nesterov_extrapolate(novak_handle *h, void *const *out, void *hip_stream);

/* Eq. 30-31 over all tensors in one launch: theta <- slow_new, and the buffer is left equal to the
 * new slow weights.  Legal only when a sync is due. */
int novak_lookahead_sync(novak_handle *h, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): ONE complete single-pass step - what novak_create, novak_step with
 * auto_sync and novak_destroy do together - without a handle and without any allocation.  The chunk
 * table, the pointer records and the clipping pre-pass's reduction buffers live in a static device array
 * of NOVAK_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends; the
 * tables are written there by a small kernel from its arguments (64 tensors per launch), in stream order
 * before the update.  Calls no hipMalloc / hipFree / allocating library routine and copies nothing
 * from host memory.
 *   hp, tensors, grads, grad_dtype, step: as for novak_create / novak_step (host arrays of device pointers;
 *     the caller owns all tensor memory).  Supported: every single-pass option (rectification, the Nesterov
 *     variants, decay, bf16 gradients / first moment, clipping, sparse threshold, lookahead with
 *     auto_sync = 1).  layer_adaptation, auto_lr, use_gc (after the fast-path downgrade) return
 *     NOVAK_ERR_NOT_IMPLEMENTED; lookahead with auto_sync = 0 returns NOVAK_ERR_INVALID_ARG.
 *   Limits: n_tensors <= NOVAK_STATIC_MAX_TENSORS and at most NOVAK_STATIC_MAX_CHUNKS chunk-table entries
 *     (sum over tensors of ceil(numel / 16384), i.e. up to 2^29 elements; with clipping the entry size follows the
 *     rule of NOVAK_TUNE_CHUNK_ELEMS, the same as a handle's, and may be 65536 or 4096); beyond them NOVAK_ERR_INVALID_ARG.
 *   No state is kept between calls: `step` is not checked against an earlier call, and the lookahead buffers
 *     must have been initialised by the caller (copy of theta) before the first step of the first window.
 *   All calls on one GPU share that GPU's array.  A call writes every entry it later reads, so nothing
 *     depends on the previous call's contents and nothing needs clearing; but two calls whose kernels may
 *     run at the same time on one GPU (different streams without an event dependency) race on it.
 *   Errors are reported through the return code and novak_last_error(NULL). */
#define NOVAK_STATIC_MAX_TENSORS 1024
#define NOVAK_STATIC_MAX_CHUNKS 32768
#define NOVAK_STATIC_SCRATCH_BYTES (2u << 20)
int novak_step_static(const novak_hparams *hp, const novak_tensor_desc *tensors, int32_t n_tensors, void *const *grads,
                      int32_t grad_dtype, int64_t step, int32_t device_id, void *hip_stream);

/* End of Algorithm 1's loop: frees the handle and its tables.  The optimizer state of Table 3 (theta, m,
 * v, lookahead buffer) is the caller's and is untouched; together with the step count it is all that
 * resuming needs.  Waits for nothing: the caller synchronises its stream first.  NULL is a no-op. */
int novak_destroy(novak_handle *h);

int novak_get_info(const novak_handle *h, novak_info *info);

/* Adjusts a launch parameter (NOVAK_TUNE_*); rebuilds the chunk table when needed (that waits for the
 * device).  It takes no stream: call it when the handle's earlier steps have finished (synchronise their
 * stream first).  Results do not depend on tuning values.  The bfloat16-moment, the centralizing and the adaptive-beta step
 * kernels exist only in the default launch shape and ignore THREADS / VEC_PER_LANE.  If a table rebuild fails
 * after the old tables were released, the handle keeps none: every later call on it but novak_destroy,
 * novak_get_info and novak_last_error returns NOVAK_ERR_STATE. */
int novak_set_tuning(novak_handle *h, int32_t key, int64_t value);

/* Text of the most recent failure on this handle (or of the last failed novak_create on this
 * thread when h is NULL).  Never NULL; valid until the next call on the same handle/thread. */
const char *novak_last_error(const novak_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* NOVAK_H_ */
