// HIP kernels of the NOVAK update-step library for gfx950 (MI355X): the fused single-pass update over
// a multi-tensor chunk table, the lookahead sync / init kernels, the Eq. 10 extrapolation, and the
// two-pass path with its norm reductions, clipping and centralization pre-passes.
// Included once, by novak_device.hip, which holds the handle and the C entry points.
//
// The step is HBM-bound (section 5.5 of the paper: 4 streams read, 3 written per element, a few
// dozen flops), so the kernels are built around memory streams, not arithmetic:
//   * a chunk-table entry never spans tensors and is covered by short-lived workgroups (one wave64
//     by default) that each touch 256..4096 consecutive elements once;
//   * each lane moves 128 bits per stream per access (4 fp32; 4 bf16 values = 64 bits), and all
//     loads of a workgroup are issued before any arithmetic;
//   * per-step scalars arrive as kernel arguments (SGPRs); nothing is read from memory except the
//     chunk entry, the tensor's pointer record and the streams themselves;
//   * streams are touched exactly once per step, so loads and stores may carry non-temporal hints.
// Arithmetic is IEEE fp32 with explicit FMAs (compiled with -ffp-contract=off, no fast-math);
// square root and division are the correctly rounded ones.
#ifndef NOVAK_KERNELS_H_
#define NOVAK_KERNELS_H_

#include <hip/hip_runtime.h>

#include <cstdint>

#include "novak_internal.h"
#include "novak_prologue.h"

namespace {

constexpr int kMinSub = 64 * 4;   // elements covered by the smallest workgroup (one wave64, one 128-bit access per lane)

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

// lookahead work done inside the step kernel (which extra stream is read / written)
enum : int {
  LA_OFF = 0,          // no lookahead traffic in this step
  LA_FIRST = 1,        // first step of a window:  A  = c0*theta_in + c1*theta_new      (A written)
  LA_MID = 2,          // later steps:             A += c1*theta_new                    (A read, written)
  LA_LAST_FUSED = 3,   // k-th step, sync fused:   theta_out = A + c1*theta_new         (A read)
  LA_BASIC_FUSED = 4,  // k-th step, basic mode:   S = c1*theta_new + c0*S; theta_out=S (S read, written)
  // template arguments only (device-step mode): the phase is a run-time, wave-uniform value
  LA_RUNTIME_ME = 5,   // one of LA_FIRST / LA_MID / LA_LAST_FUSED
  LA_RUNTIME_BASIC = 6 // LA_OFF or LA_BASIC_FUSED
};
constexpr bool la_runtime(int la) { return la >= LA_RUNTIME_ME; }

enum : uint32_t {
  F_APPROX = 1u, F_CLASSICAL = 2u, F_DENOM = 4u, F_COUPLED = 8u, F_CLIP = 16u, F_SPARSE = 32u, F_GC = 64u, F_AUTO = 128u,
  F_LITERAL_M = 256u, F_LITERAL_V = 512u   // adaptive-beta kernels only: this step evaluates Eq. 1 / Eq. 2 as printed
};

// The four state pointers of a tensor sit together so that one 32-byte scalar load fetches them.
struct TensorPtrs {
  float *param;
  float *m;
  float *v;
  float *la;
};

// Gradient centralization (Eq. 26) of one tensor: rows of `cols` contiguous elements; cols == 0 means
// the tensor is not centralized.  `means` holds this step's mean of every row of the raw gradient, in
// double: g - mean is formed in double and rounded once, so an element whose centralized gradient
// nearly cancels keeps a relative (not absolute) error - at t = 1 the direction g/(|g|+eps) is
// sign-like and would amplify an absolute error of half an ulp of g.
struct GcInfo {
  int64_t cols;
  double inv_cols;
  const double *means;
};

struct Tables {
  const novak_chunk *chunks;
  const TensorPtrs *tensors;
  const void *const *grad;
  const float *gscale;   // one float: the step's gradient-clipping factor (read only when F_CLIP is set)
  const GcInfo *gc;      // per tensor (read only when F_GC is set)
  const float *ascale;   // one float: the step's auto-LR factor of Eq. 22 (read only when F_AUTO is set: auto-LR without
                         // a trust ratio needs global norms only, which a pre-pass supplies to the single-pass step)
};

// idx / cols for 0 <= idx < 2^52 without an integer divide: double estimate, then one correction step
__device__ __forceinline__ int64_t row_of(int64_t idx, int64_t cols, double inv_cols) {
  int64_t q = static_cast<int64_t>(static_cast<double>(idx) * inv_cols);
  if (q * cols > idx) --q;
  else if ((q + 1) * cols <= idx) ++q;
  return q;
}

// Subtracts the row means from `n` (<= 4) consecutive gradient values that start at element `e0` of a
// centralized tensor.  Centralizing the raw gradient and scaling by the clipping factor afterwards
// equals clipping first (the factor is one scalar for all tensors).
template <typename V>
__device__ __forceinline__ void centralize(V &g, int n, int64_t e0, const GcInfo &gc) {
  int64_t row = row_of(e0, gc.cols, gc.inv_cols);
  int64_t rem = e0 - row * gc.cols;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (k < n) {
      while (rem >= gc.cols) { rem -= gc.cols; ++row; }
      g[k] = static_cast<float>(static_cast<double>(g[k]) - gc.means[row]);
      ++rem;
    }
  }
}
__device__ __forceinline__ float centralize_one(float g, int64_t e, const GcInfo &gc) {
  return static_cast<float>(static_cast<double>(g) - gc.means[row_of(e, gc.cols, gc.inv_cols)]);
}

// Per-step scalars, rounded once from the host's double values.
struct Consts {
  float omb1, omb2;      // 1-beta1, 1-beta2
  float beta1, beta_n;
  float inv_bc1, inv_bc2;
  float eps;
  float step_size;       // alpha * r_t
  float lr_wd;           // alpha * lambda (decoupled) or 0
  float wd;              // lambda (coupled) or 0
  float la_c0, la_c1;    // lookahead blend coefficients (meaning depends on the LA phase)
  float sparse_tau;      // tau of Eq. 27 (used when F_SPARSE is set)
  float blend_w;         // 1-beta1 of Eq. 16 (base beta1; omb1 follows the schedule of Eq. 3)
  float beta1_t, beta2_t;  // the scheduled betas of Eq. 3-4 (read by the adaptive-beta kernels only)
  uint32_t flags;
};

// Device-step mode: what one step is, written by novak_prologue_kernel, read by the step's kernels.  The records of
// up to kDeviceRing consecutive steps sit side by side (one per 128 bytes).
constexpr int kDeviceRing = 64;
struct DeviceStep {
  Consts c;
  int la;              // LA_* phase of this step
  int64_t t;           // the step's number
  int64_t *counter;    // the caller's step counter: the step's last kernel stores t there
  int pad[10];
};
static_assert(sizeof(DeviceStep) == 128, "one record per 128 bytes");

// One lane of the step's last kernel records that step d.t has been taken.
__device__ __forceinline__ void device_step_done(const DeviceStep &d) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *d.counter = d.t;
}

__device__ __forceinline__ float bf16_to_f32(unsigned short b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// fp32 -> bfloat16, round to nearest even; NaN stays NaN (quiet), infinities stay
__device__ __forceinline__ unsigned short f32_to_bf16(float x) {
  uint32_t b = __float_as_uint(x);
  if ((b & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((b >> 16) | 0x40u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return static_cast<unsigned short>(b >> 16);
}

// The first moment as stored: fp32, or bfloat16 (rounded once per step from the fp32 value of Eq. 1).
// store_m returns what was stored, which is the m_t the rest of the step uses.
template <typename MomV>
__device__ __forceinline__ f32x4 mom_to_f32(MomV m);
template <>
__device__ __forceinline__ f32x4 mom_to_f32<f32x4>(f32x4 m) { return m; }
template <>
__device__ __forceinline__ f32x4 mom_to_f32<u16x4>(u16x4 m) {
  f32x4 r;
#pragma unroll
  for (int k = 0; k < 4; ++k) r[k] = bf16_to_f32(m[k]);
  return r;
}
template <typename MomS>
__device__ __forceinline__ float round_mom(float m) {
  if constexpr (sizeof(MomS) == 2) return bf16_to_f32(f32_to_bf16(m));
  else return m;
}
template <typename MomV>
__device__ __forceinline__ MomV f32_to_mom(f32x4 m);
template <>
__device__ __forceinline__ f32x4 f32_to_mom<f32x4>(f32x4 m) { return m; }
template <>
__device__ __forceinline__ u16x4 f32_to_mom<u16x4>(f32x4 m) {
  u16x4 r;
#pragma unroll
  for (int k = 0; k < 4; ++k) r[k] = f32_to_bf16(m[k]);
  return r;
}
template <typename MomS>
__device__ __forceinline__ float load_mom(const MomS *p) {
  if constexpr (sizeof(MomS) == 2) return bf16_to_f32(*p);
  else return *p;
}
template <typename MomS>
__device__ __forceinline__ void store_mom(MomS *p, float m) {
  if constexpr (sizeof(MomS) == 2) *p = f32_to_bf16(m);
  else *p = m;
}

// The update of one element, in three parts so that the two-pass (per-tensor scaled) path can reuse
// the exact arithmetic of the fused one.
//   moments():   Phases 2 and 4 - gradient processing and the two EMAs (Eq. 13, 1, 2)
//   direction(): Phases 5 and 8a - bias correction and the base direction u (Eq. 5, 17)
//   apply():     Phases 8b, 9, 10 - classical blend, decay + update, lookahead (Eq. 16, 18, 24, 28-31)
// AB: compiled for handles with the adaptive-beta schedule of Eq. 3-4, whose betas start near 0.  There the
// difference form rounds at the magnitude of the OLD moment although the new one is ~beta(t) times smaller (an element
// whose gradient has dropped keeps a relative error of 2^-24 / beta(t)), so while beta(t) <= 1/2 Eq. 1-2 are evaluated
// as printed (the rounding of beta and 1 - beta, which do not add up to 1 exactly, is amplified by at most 2 there).
template <bool AB = false>
__device__ __forceinline__ void moments(float th_in, float g, float &m, float &v, const Consts &c, float gs) {
  if (c.flags & F_CLIP) g *= gs;                                        // global-norm clipping comes first
  if (c.flags & F_COUPLED) g = __builtin_fmaf(c.wd, th_in, g);          // classic L2 reading
  if (c.flags & F_APPROX) g = __builtin_fmaf(c.beta_n, g - m, g);       // Eq. 13
  const float m_in = m, v_in = v;
  m = __builtin_fmaf(c.omb1, g - m, m);                                 // Eq. 1:  m + (1-b1)(g - m)
  v = __builtin_fmaf(c.omb2, __builtin_fmaf(g, g, -v), v);              // Eq. 2:  v + (1-b2)(g^2 - v)
  if constexpr (AB) {
    if (c.flags & F_LITERAL_M) m = __builtin_fmaf(c.omb1, g, c.beta1_t * m_in);        // Eq. 1 as printed
    if (c.flags & F_LITERAL_V) v = __builtin_fmaf(c.omb2, g * g, c.beta2_t * v_in);    // Eq. 2 as printed
  }
  // A moment that has overflowed stays infinite under Eq. 1-2 as printed (beta*inf + finite); the
  // difference form above would turn it into inf - inf.  With v = inf the direction is 0 and theta only decays.
  const bool g_finite = __builtin_fabsf(g) < __builtin_inff();
  if (__builtin_isinf(m_in) && g_finite) m = m_in;
  if (__builtin_isinf(v_in) && g == g) v = v_in;
}

__device__ __forceinline__ float direction(float m, float v, const Consts &c, float &m_hat) {
  m_hat = m * c.inv_bc1;                                                // Eq. 5
  float u = m_hat;
  if (c.flags & F_DENOM) {
    const float v_hat = v * c.inv_bc2;                                  // Eq. 5
    u = m_hat / (__builtin_sqrtf(v_hat) + c.eps);                       // Eq. 17
  }
  return u;
}

// `step` is alpha*r_t, times the tensor's trust ratio and the auto-LR factor on the scaled path (Eq. 24a).
// `la` is the lookahead buffer value (read when the phase reads it, returned updated when it writes it).
template <int LA>
__device__ __forceinline__ void apply(float &th, float u, float m_hat, float &la, const Consts &c, float step, int la_rt = LA_OFF) {
  const float th_in = th;
  if ((c.flags & F_SPARSE) && !(__builtin_fabsf(u) > c.sparse_tau)) u = 0.0f;  // Eq. 27
  if (c.flags & F_CLASSICAL) u = __builtin_fmaf(c.beta1, m_hat, c.blend_w * u);  // Eq. 16
  // Eq. 18 + Eq. 24 in additive form: one rounding at theta's magnitude per step
  const float th_new = th_in - __builtin_fmaf(step, u, c.lr_wd * th_in);
  th = th_new;
  if (LA == LA_FIRST) {
    la = __builtin_fmaf(c.la_c1, th_new, c.la_c0 * th_in);
  } else if (LA == LA_MID) {
    la = __builtin_fmaf(c.la_c1, th_new, la);
  } else if (LA == LA_LAST_FUSED) {
    th = __builtin_fmaf(c.la_c1, th_new, la);                           // Eq. 30-31
  } else if (LA == LA_BASIC_FUSED) {
    la = __builtin_fmaf(c.la_c1, th_new, c.la_c0 * la);
    th = la;
  } else if (la_runtime(LA)) {
    // the same expressions, selected by a wave-uniform phase: results are bit-identical to the compiled-in phases
    const float la_in = la;
    const float scaled = c.la_c0 * (la_rt == LA_FIRST ? th_in : la_in);
    const float base = (la_rt == LA_FIRST || la_rt == LA_BASIC_FUSED) ? scaled : la_in;
    const float blend = __builtin_fmaf(c.la_c1, th_new, base);
    if (la_rt == LA_FIRST || la_rt == LA_MID || la_rt == LA_BASIC_FUSED) la = blend;
    if (la_rt == LA_LAST_FUSED || la_rt == LA_BASIC_FUSED) th = blend;
  }
}

template <int LA, typename MomS = float, bool AB = false>
__device__ __forceinline__ void update_one(float &th, float g, float &m, float &v, float &la, const Consts &c, float gs, float step, int la_rt = LA_OFF) {
  moments<AB>(th, g, m, v, c, gs);
  m = round_mom<MomS>(m);          // the stored m_t is what the rest of the step uses
  float m_hat;
  const float u = direction(m, v, c, m_hat);
  apply<LA>(th, u, m_hat, la, c, step, la_rt);
}

// Vector loads and stores of tensor data.  Every tensor pointer is device (global) memory, which the compiler cannot
// know of a pointer it read from a table: said here, so that it emits global_load / global_store (results return in
// issue order, and a wait can name how many later loads may stay in flight) instead of flat accesses.
#define NOVAK_GLOBAL __attribute__((address_space(1)))
template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *p) {
  const NOVAK_GLOBAL T *q = (const NOVAK_GLOBAL T *)p;
  if (NT) return __builtin_nontemporal_load(q);
  return *q;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T *p, T x) {
  NOVAK_GLOBAL T *q = (NOVAK_GLOBAL T *)p;
  if (NT) __builtin_nontemporal_store(x, q);
  else *q = x;
}

// The row means that 4 consecutive elements starting at e0 need, for rows of at least 4 elements (then the 4 lie in at
// most two rows): both loads are unconditional, so they can be issued together with the step's own loads, before any
// gradient value has arrived.  (Behind the branches of `centralize` the loads waited for the gradient wherever it has
// to be converted first: the bfloat16-gradient kernels paid a second memory round trip per wave, 12-14 % of their time.)
struct RowMeans4 {
  double first, second;   // mean of the row of element e0, and of the next row if the 4 elements reach into it
  int split;              // elements k < split belong to the first row
};
__device__ __forceinline__ RowMeans4 load_row_means(int64_t e0, const GcInfo &gc) {
  const int64_t row = row_of(e0, gc.cols, gc.inv_cols);
  const int64_t left = (row + 1) * gc.cols - e0;          // elements of that row from e0 on (>= 1)
  const NOVAK_GLOBAL double *means = (const NOVAK_GLOBAL double *)gc.means;
  RowMeans4 r;
  r.split = left < 4 ? static_cast<int>(left) : 4;
  r.first = means[row];
  r.second = means[row + (left < 4 ? 1 : 0)];
  return r;
}
template <typename V>
__device__ __forceinline__ void centralize4(V &g, const RowMeans4 &r) {
#pragma unroll
  for (int k = 0; k < 4; ++k) g[k] = static_cast<float>(static_cast<double>(g[k]) - (k < r.split ? r.first : r.second));
}

template <typename GradV>
__device__ __forceinline__ f32x4 grad_to_f32(GradV g);
template <>
__device__ __forceinline__ f32x4 grad_to_f32<f32x4>(f32x4 g) { return g; }
template <>
__device__ __forceinline__ f32x4 grad_to_f32<u16x4>(u16x4 g) {
  f32x4 r;
#pragma unroll
  for (int k = 0; k < 4; ++k) r[k] = bf16_to_f32(g[k]);
  return r;
}

template <int LA, typename MomS = float, bool AB = false>
__device__ __forceinline__ void update_vec(f32x4 &th, f32x4 g, f32x4 &m, f32x4 &v, f32x4 &la, const Consts &c, float gs, float step, int la_rt = LA_OFF) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float th_k = th[k], m_k = m[k], v_k = v[k], la_k = la[k];
    update_one<LA, MomS, AB>(th_k, g[k], m_k, v_k, la_k, c, gs, step, la_rt);
    th[k] = th_k; m[k] = m_k; v[k] = v_k; la[k] = la_k;
  }
}

__host__ __device__ constexpr bool la_reads(int la) { return la == LA_MID || la == LA_LAST_FUSED || la == LA_BASIC_FUSED; }
__host__ __device__ constexpr bool la_writes(int la) { return la == LA_FIRST || la == LA_MID || la == LA_BASIC_FUSED; }

// Work decomposition.  A chunk-table entry covers up to chunk_elems (a power of two) elements of one
// tensor; it is processed by chunk_elems / SUB workgroups ("sub-blocks"), each of which touches
// SUB = BLOCK*4*UN consecutive elements exactly once and exits.  The default is BLOCK = 64, UN = 1:
// one wave64 per 256 elements, one 128-bit access per lane and stream.  Short-lived workgroups dispatched
// in address order keep the set of DRAM pages that are open at any moment small, which is what the
// write path of this memory system rewards; the table stays small because its granularity is
// decoupled from the workgroup's.  blockIdx.x = (chunk index << sub_shift) | sub-block index.
//
// GradS: scalar gradient type (float, or unsigned short holding bf16 bits); GradV its 4-vector.
// GC: compiled-in gradient centralization (Eq. 26) for tensors that ask for it (only instantiated for
// the default shape UN = 1, BLOCK = 64).
// MomS / MomV: storage type of the first moment and its 4-vector (float / f32x4, or unsigned short /
// u16x4 for bfloat16; the latter also only for UN = 1, BLOCK = 64).
// AB: the adaptive-beta variant of the moment updates (see moments; also only for UN = 1, BLOCK = 64).
template <typename GradS, typename GradV, int LA, bool NT, int UN, int BLOCK, bool GC = false, typename MomS = float,
          typename MomV = f32x4, bool DEV = false, bool AB = false>
__device__ __forceinline__ void step_body(const Tables &tb, const Consts &c_arg, int sub_shift, const DeviceStep *ds = nullptr) {
  constexpr int SUB = BLOCK * 4 * UN;
  const novak_chunk ch = tb.chunks[blockIdx.x >> sub_shift];
  const int start = static_cast<int>(blockIdx.x & ((1u << sub_shift) - 1u)) * SUB;
  if (start >= ch.len) return;
  const int n = min(SUB, ch.len - start);
  const int64_t off = ch.offset + start;
  const TensorPtrs tp = tb.tensors[ch.tensor];          // one scalar load, issued together with the next
  const void *const g_base = tb.grad[ch.tensor];
  // Device-step mode (DEV): constants and lookahead phase come from device memory; their scalar load is issued
  // here, together with the two table loads above, so that the wave waits once for all three.
  DeviceStep d;
  if constexpr (DEV) d = *ds;
  const Consts &c = DEV ? d.c : c_arg;
  // which lookahead stream this step reads / writes: compiled in, or a wave-uniform run-time value
  const int la_rt = DEV ? d.la : LA_OFF;
  const int phase = la_runtime(LA) ? la_rt : LA;
  const bool reads = la_reads(phase), writes = la_writes(phase);
  const float gs = (c.flags & F_CLIP) ? *tb.gscale : 1.0f;
  const float step = (c.flags & F_AUTO) ? c.step_size * *tb.ascale : c.step_size;     // Eq. 24a with lambda_trust = 1
  GcInfo gi;
  gi.cols = 0;
  if (GC) gi = tb.gc[ch.tensor];
  // The counter's store comes after every wave-uniform load: behind a store that may alias them the compiler reads
  // such values with vector loads and waits for them together with the step's own loads (the centralizing device-step
  // kernels then issued the row-mean loads a memory round trip late: -7 ... -9 %).
  if constexpr (DEV) device_step_done(d);
  float *__restrict__ th_p = tp.param + off;
  MomS *__restrict__ m_p = reinterpret_cast<MomS *>(tp.m) + off;
  float *__restrict__ v_p = tp.v + off;
  const GradS *__restrict__ g_p = static_cast<const GradS *>(g_base) + off;
  float *__restrict__ la_p = nullptr;
  if (phase != LA_OFF) la_p = tp.la + off;

  uintptr_t mis = (reinterpret_cast<uintptr_t>(th_p) | reinterpret_cast<uintptr_t>(v_p) | reinterpret_cast<uintptr_t>(la_p)) & 15u;
  mis |= reinterpret_cast<uintptr_t>(g_p) & (sizeof(GradV) - 1);
  mis |= reinterpret_cast<uintptr_t>(m_p) & (sizeof(MomV) - 1);

  int done = 0;   // elements [0, done) handled by the 128-bit path
  if (mis == 0) {
    f32x4 *th4 = reinterpret_cast<f32x4 *>(th_p);
    MomV *m4 = reinterpret_cast<MomV *>(m_p);
    f32x4 *v4 = reinterpret_cast<f32x4 *>(v_p);
    f32x4 *la4 = reinterpret_cast<f32x4 *>(la_p);
    const GradV *g4 = reinterpret_cast<const GradV *>(g_p);
    if (n == SUB) {
      // full sub-block: every load is issued before any arithmetic.  With a run-time phase the lookahead load is
      // issued whatever the phase (behind a uniform branch it was issued late: -9 ... -13 %): from the buffer when
      // the phase reads it, else from theta's own address, whose line is on its way already.
      const f32x4 *la_src = (la_runtime(LA) && !reads) ? th4 : la4;
      const bool load_la = la_runtime(LA) ? true : reads;
      f32x4 th[UN], v[UN], la[UN];
      MomV m[UN];
      GradV g[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int j = threadIdx.x + u * BLOCK;
        th[u] = ld<NT>(th4 + j);
        g[u] = ld<NT>(g4 + j);
        m[u] = ld<NT>(m4 + j);
        v[u] = ld<NT>(v4 + j);
        if (load_la) la[u] = ld<NT>(la_src + j);
      }
      RowMeans4 rm[UN];
      if (GC && gi.cols >= 4) {
#pragma unroll
        for (int u = 0; u < UN; ++u) rm[u] = load_row_means(off + 4 * static_cast<int64_t>(threadIdx.x + u * BLOCK), gi);
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int j = threadIdx.x + u * BLOCK;
        f32x4 gf = grad_to_f32<GradV>(g[u]);
        if (GC && gi.cols >= 4) centralize4(gf, rm[u]);
        else if (GC && gi.cols) centralize(gf, 4, off + 4 * static_cast<int64_t>(j), gi);
        f32x4 mf = mom_to_f32<MomV>(m[u]);
        update_vec<LA, MomS, AB>(th[u], gf, mf, v[u], la[u], c, gs, step, la_rt);
        st<NT>(th4 + j, th[u]);
        st<NT>(m4 + j, f32_to_mom<MomV>(mf));
        st<NT>(v4 + j, v[u]);
        if (writes) st<NT>(la4 + j, la[u]);
      }
      return;
    }
    const int nvec = n >> 2;
    for (int i = threadIdx.x; i < nvec; i += BLOCK) {
      f32x4 th = ld<NT>(th4 + i), m = mom_to_f32<MomV>(ld<NT>(m4 + i)), v = ld<NT>(v4 + i), la;
      GradV g = ld<NT>(g4 + i);
      if (reads) la = ld<NT>(la4 + i);
      RowMeans4 rm;
      if (GC && gi.cols >= 4) rm = load_row_means(off + 4 * static_cast<int64_t>(i), gi);
      f32x4 gf = grad_to_f32<GradV>(g);
      if (GC && gi.cols >= 4) centralize4(gf, rm);
      else if (GC && gi.cols) centralize(gf, 4, off + 4 * static_cast<int64_t>(i), gi);
      update_vec<LA, MomS, AB>(th, gf, m, v, la, c, gs, step, la_rt);
      st<NT>(th4 + i, th);
      st<NT>(m4 + i, f32_to_mom<MomV>(m));
      st<NT>(v4 + i, v);
      if (writes) st<NT>(la4 + i, la);
    }
    done = nvec << 2;
  }
  // element-wise path: the < 4 element tail of an aligned sub-block, or a whole unaligned one
  for (int i = done + threadIdx.x; i < n; i += BLOCK) {
    float th = th_p[i], m = load_mom<MomS>(m_p + i), v = v_p[i], la = 0.0f, g;
    if constexpr (sizeof(GradS) == 2) g = bf16_to_f32(g_p[i]);
    else g = g_p[i];
    if (reads) la = la_p[i];
    if (GC && gi.cols) g = centralize_one(g, off + i, gi);
    update_one<LA, MomS, AB>(th, g, m, v, la, c, gs, step, la_rt);
    th_p[i] = th;
    store_mom<MomS>(m_p + i, m);
    v_p[i] = v;
    if (writes) la_p[i] = la;
  }
}

template <typename GradS, typename GradV, int LA, bool NT, int UN, int BLOCK, bool GC = false, typename MomS = float,
          typename MomV = f32x4, bool AB = false>
__global__ __launch_bounds__(BLOCK) void novak_step_kernel(Tables tb, Consts c, int sub_shift) {
  step_body<GradS, GradV, LA, NT, UN, BLOCK, GC, MomS, MomV, false, AB>(tb, c, sub_shift);
}

// Device-step mode: what the step is (constants, lookahead phase) was written to device memory by
// novak_prologue_kernel just before; every wave fetches it with one scalar load.  LA is LA_OFF (no lookahead),
// LA_RUNTIME_ME or LA_RUNTIME_BASIC: one body in which the lookahead blend and store are selected by the wave-uniform
// phase (compiling the phase bodies behind a switch made the compiler merge them and lose the "all loads first"
// order: -10 %).  Default launch shape only (one wave64 per 256 elements).
template <typename GradS, typename GradV, int LA, bool NT, bool GC, typename MomS, typename MomV, bool AB>
__global__ __launch_bounds__(64) void novak_step_device_kernel(Tables tb, const DeviceStep *ds, int sub_shift) {
  step_body<GradS, GradV, LA, NT, 1, 64, GC, MomS, MomV, true, AB>(tb, Consts(), sub_shift, ds);
}

// What step t does: the kernel constants (scalar prologue of Phases 5-6 rounded to fp32) and the lookahead
// phase of the step (its position in the k-step window of section 4.7).  Evaluated on the host by novak_step, and
// by novak_prologue_kernel on the device in device-step mode.
struct StepPlan {
  Consts c;
  int la = LA_OFF;
  bool window_closes = false;   // t mod k == 0
  bool sync_after = false;      // k == 1 with auto_sync: the sync cannot be fused into a later step of the window
};

__host__ __device__ inline void plan_step(const novak_hparams &hp, int64_t step, StepPlan *pl) {
  novak_step_scalars sc;
  novak_step_scalars_impl(hp, step, &sc);
  Consts c = Consts();
  c.omb1 = static_cast<float>(1.0 - sc.beta1_t);      // the moment updates follow Eq. 3-4 when scheduled
  c.omb2 = static_cast<float>(1.0 - sc.beta2_t);
  c.beta1_t = static_cast<float>(sc.beta1_t);
  c.beta2_t = static_cast<float>(sc.beta2_t);
  c.blend_w = static_cast<float>(1.0 - hp.beta1);
  c.beta1 = static_cast<float>(hp.beta1);
  c.beta_n = static_cast<float>(hp.beta_n);
  c.inv_bc1 = static_cast<float>(1.0 / sc.bc1);
  c.inv_bc2 = static_cast<float>(1.0 / sc.bc2);
  c.eps = static_cast<float>(hp.eps);
  c.step_size = static_cast<float>(sc.step_size);
  c.lr_wd = hp.decoupled_decay ? static_cast<float>(hp.lr * hp.weight_decay) : 0.0f;
  c.wd = hp.decoupled_decay ? 0.0f : static_cast<float>(hp.weight_decay);
  c.flags = 0;
  if (sc.nesterov_mode == NOVAK_NESTEROV_APPROX) c.flags |= F_APPROX;
  if (hp.nesterov_mode == NOVAK_NESTEROV_CLASSICAL) c.flags |= F_CLASSICAL;
  if (sc.denom_on) c.flags |= F_DENOM;
  if (!hp.decoupled_decay && hp.weight_decay != 0.0) c.flags |= F_COUPLED;
  if (hp.clip_threshold > 0.0) c.flags |= F_CLIP;
  if (hp.adaptive_beta && sc.beta1_t <= 0.5) c.flags |= F_LITERAL_M;
  if (hp.adaptive_beta && sc.beta2_t <= 0.5) c.flags |= F_LITERAL_V;
  if (hp.sparse_threshold > 0.0) {
    c.flags |= F_SPARSE;
    c.sparse_tau = static_cast<float>(hp.sparse_threshold);
  }
  // lookahead phase of this step: position in the k-step window (section 4.7; sync when t mod k == 0)
  pl->la = LA_OFF;
  pl->window_closes = pl->sync_after = false;
  if (hp.lookahead_mode != NOVAK_LOOKAHEAD_NONE) {
    const int64_t pos = (step - 1) % hp.la_k + 1;
    pl->window_closes = pos == hp.la_k;
    if (hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT) {
      c.la_c0 = static_cast<float>(1.0 - hp.la_alpha);
      c.la_c1 = static_cast<float>(hp.la_alpha / hp.la_k);
      if (pos == 1) {
        pl->la = LA_FIRST;
        pl->sync_after = pl->window_closes && hp.auto_sync;   // k == 1: nothing to fuse into
      } else if (pl->window_closes && hp.auto_sync) {
        pl->la = LA_LAST_FUSED;
      } else {
        pl->la = LA_MID;
      }
    } else if (pl->window_closes && hp.auto_sync) {
      pl->la = LA_BASIC_FUSED;
      c.la_c0 = static_cast<float>(1.0 - hp.la_alpha);
      c.la_c1 = static_cast<float>(hp.la_alpha);
    }
  }
  pl->c = c;
}

// Device-step mode: lane i writes what step counter + 1 + i is, for i < count <= kDeviceRing.  The counter itself is
// advanced by the steps: the last kernel of each stores its t there (device_step_done).
__global__ __launch_bounds__(kDeviceRing) void novak_prologue_kernel(novak_hparams hp, uint32_t extra_flags, int64_t *counter, DeviceStep *out, int count) {
  if (static_cast<int>(threadIdx.x) >= count) return;
  const int64_t t = *counter + 1 + threadIdx.x;
  StepPlan pl;
  plan_step(hp, t, &pl);
  DeviceStep d;
  d.c = pl.c;
  d.c.flags |= extra_flags;
  d.la = pl.la;
  d.t = t;
  d.counter = counter;
#pragma unroll
  for (int i = 0; i < 10; ++i) d.pad[i] = 0;
  out[threadIdx.x] = d;
}

// A list without elements launches no kernel that could do it.
__global__ __launch_bounds__(64) void novak_count_kernel(const DeviceStep *ds) {
  device_step_done(*ds);
}

// Lookahead kernels over the same chunk table and sub-block decomposition (UN = 1).
//   SYNC_ME:    theta <- A                       (A already holds Eq. 30's right-hand side)
//   SYNC_BASIC: S <- c1*theta + c0*S; theta <- S (standard Lookahead interpolation)
//   INIT:       buffer <- theta                  (Eq. 28)
enum : int { SYNC_ME = 0, SYNC_BASIC = 1, LA_INIT = 2 };

template <int OP>
__device__ __forceinline__ void la_one(float &th, float &la, float c0, float c1) {
  if (OP == SYNC_ME) th = la;
  else if (OP == SYNC_BASIC) { la = __builtin_fmaf(c1, th, c0 * la); th = la; }
  else la = th;
}

template <int OP, bool NT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void novak_lookahead_kernel(Tables tb, float c0, float c1, int sub_shift) {
  constexpr int SUB = BLOCK * 4;
  const novak_chunk ch = tb.chunks[blockIdx.x >> sub_shift];
  const int start = static_cast<int>(blockIdx.x & ((1u << sub_shift) - 1u)) * SUB;
  if (start >= ch.len) return;
  const int n = min(SUB, ch.len - start);
  const int64_t off = ch.offset + start;
  const TensorPtrs tp = tb.tensors[ch.tensor];
  float *__restrict__ th_p = tp.param + off;
  float *__restrict__ la_p = tp.la + off;
  const uintptr_t mis = (reinterpret_cast<uintptr_t>(th_p) | reinterpret_cast<uintptr_t>(la_p)) & 15u;
  int done = 0;
  if (mis == 0) {
    const int nvec = n >> 2;
    f32x4 *th4 = reinterpret_cast<f32x4 *>(th_p);
    f32x4 *la4 = reinterpret_cast<f32x4 *>(la_p);
    for (int i = threadIdx.x; i < nvec; i += BLOCK) {
      f32x4 th, la;
      if (OP != SYNC_ME) th = ld<NT>(th4 + i);
      if (OP != LA_INIT) la = ld<NT>(la4 + i);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float th_k = th[k], la_k = la[k];
        la_one<OP>(th_k, la_k, c0, c1);
        th[k] = th_k; la[k] = la_k;
      }
      if (OP != LA_INIT) st<NT>(th4 + i, th);
      if (OP != SYNC_ME) st<NT>(la4 + i, la);
    }
    done = nvec << 2;
  }
  for (int i = done + threadIdx.x; i < n; i += BLOCK) {
    float th = 0.0f, la = 0.0f;
    if (OP != SYNC_ME) th = th_p[i];
    if (OP != LA_INIT) la = la_p[i];
    la_one<OP>(th, la, c0, c1);
    if (OP != LA_INIT) th_p[i] = th;
    if (OP != SYNC_ME) la_p[i] = la;
  }
}

// True Nesterov, Eq. 10: out <- theta + beta_n * m over the chunk table (one wave per 256 elements).
template <bool NT, typename MomS = float, typename MomV = f32x4>
__global__ __launch_bounds__(64) void novak_extrapolate_kernel(Tables tb, float *const *out, float beta_n, int sub_shift) {
  constexpr int SUB = 64 * 4;
  const novak_chunk ch = tb.chunks[blockIdx.x >> sub_shift];
  const int start = static_cast<int>(blockIdx.x & ((1u << sub_shift) - 1u)) * SUB;
  if (start >= ch.len) return;
  const int n = min(SUB, ch.len - start);
  const int64_t off = ch.offset + start;
  const TensorPtrs tp = tb.tensors[ch.tensor];
  const float *__restrict__ th_p = tp.param + off;
  const MomS *__restrict__ m_p = reinterpret_cast<const MomS *>(tp.m) + off;
  float *__restrict__ o_p = out[ch.tensor] + off;
  const uintptr_t mis = ((reinterpret_cast<uintptr_t>(th_p) | reinterpret_cast<uintptr_t>(o_p)) & 15u) |
                        (reinterpret_cast<uintptr_t>(m_p) & (sizeof(MomV) - 1));
  int done = 0;
  if (mis == 0) {
    const int nvec = n >> 2;
    const int i = threadIdx.x;
    if (i < nvec) {
      const f32x4 th = ld<NT>(reinterpret_cast<const f32x4 *>(th_p) + i),
                  m = mom_to_f32<MomV>(ld<NT>(reinterpret_cast<const MomV *>(m_p) + i));
      f32x4 o;
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = __builtin_fmaf(beta_n, m[k], th[k]);
      st<NT>(reinterpret_cast<f32x4 *>(o_p) + i, o);
    }
    done = nvec << 2;
  }
  for (int i = done + threadIdx.x; i < n; i += 64) o_p[i] = __builtin_fmaf(beta_n, load_mom<MomS>(m_p + i), th_p[i]);
}

// ------------------------------------------------------------------------------------------------
// Two-pass path for the full-features scalings (layer-wise trust ratio, Eq. 19 / 25; auto-LR, Eq.
// 20-22).  Both need norms over whole tensors before any parameter may move, so the step splits:
//   pass 1  novak_moments_kernel   reads theta, g, m, v; writes m, v; one partial (sum theta^2,
//                                  sum u^2, sum g^2) per wave, u being Eq. 17's base direction
//   reduce  chunks -> tensors -> (global)   fixed-order sums in double: results do not depend on timing
//   pass 2  novak_apply_kernel     reads theta, m, v; recomputes u with the same arithmetic; applies
//                                  alpha*r_t*scale[tensor] and the lookahead phase; writes theta
// One wave64 per 256 elements in both passes, as in the fused kernel.
// ------------------------------------------------------------------------------------------------
constexpr int kScaledBlock = 64;
constexpr int kScaledSub = kScaledBlock * 4;

struct NormPartial {   // one per wave of pass 1
  float theta2, u2, g2, pad;
};
struct NormSums {      // per chunk / per tensor, in double
  double theta2, u2, g2;
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// `c_arg` holds the step's constants, or (DEV, device-step mode) `ds` points to them in device memory.
template <typename GradS, typename GradV, bool NT, typename MomS, typename MomV, bool DEV, bool AB>
__device__ __forceinline__ void moments_body(const Tables &tb, const Consts &c_arg, int sub_shift, NormPartial *partials, const DeviceStep *ds) {
  const novak_chunk ch = tb.chunks[blockIdx.x >> sub_shift];
  const int start = static_cast<int>(blockIdx.x & ((1u << sub_shift) - 1u)) * kScaledSub;
  if (start >= ch.len) return;
  const int n = min(kScaledSub, ch.len - start);
  const int64_t off = ch.offset + start;
  const TensorPtrs tp = tb.tensors[ch.tensor];
  const void *const g_base = tb.grad[ch.tensor];
  Consts c_dev;
  if constexpr (DEV) c_dev = ds->c;
  const Consts &c = DEV ? c_dev : c_arg;
  const float gs = (c.flags & F_CLIP) ? *tb.gscale : 1.0f;
  GcInfo gi;
  gi.cols = 0;
  if (c.flags & F_GC) gi = tb.gc[ch.tensor];
  const float *__restrict__ th_p = tp.param + off;
  MomS *__restrict__ m_p = reinterpret_cast<MomS *>(tp.m) + off;
  float *__restrict__ v_p = tp.v + off;
  const GradS *__restrict__ g_p = static_cast<const GradS *>(g_base) + off;

  uintptr_t mis = (reinterpret_cast<uintptr_t>(th_p) | reinterpret_cast<uintptr_t>(v_p)) & 15u;
  mis |= reinterpret_cast<uintptr_t>(g_p) & (sizeof(GradV) - 1);
  mis |= reinterpret_cast<uintptr_t>(m_p) & (sizeof(MomV) - 1);

  float s_th = 0.0f, s_u = 0.0f, s_g = 0.0f;
  int done = 0;
  if (mis == 0) {
    const int nvec = n >> 2;
    const f32x4 *th4 = reinterpret_cast<const f32x4 *>(th_p);
    MomV *m4 = reinterpret_cast<MomV *>(m_p);
    f32x4 *v4 = reinterpret_cast<f32x4 *>(v_p);
    const GradV *g4 = reinterpret_cast<const GradV *>(g_p);
    const int i = threadIdx.x;
    if (i < nvec) {
      const f32x4 th = ld<NT>(th4 + i);
      const GradV g_raw = ld<NT>(g4 + i);
      const MomV m_raw = ld<NT>(m4 + i);
      f32x4 v = ld<NT>(v4 + i);
      RowMeans4 rm;
      if (gi.cols >= 4) rm = load_row_means(off + 4 * static_cast<int64_t>(i), gi);
      f32x4 g = grad_to_f32<GradV>(g_raw);
      f32x4 m = mom_to_f32<MomV>(m_raw);
#pragma unroll
      for (int k = 0; k < 4; ++k) s_g = __builtin_fmaf(g[k], g[k], s_g);     // norm of the gradient as handed in
      if (gi.cols >= 4) centralize4(g, rm);
      else if (gi.cols) centralize(g, 4, off + 4 * static_cast<int64_t>(i), gi);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float m_k = m[k], v_k = v[k], m_hat;
        moments<AB>(th[k], g[k], m_k, v_k, c, gs);
        m_k = round_mom<MomS>(m_k);
        const float u = direction(m_k, v_k, c, m_hat);
        s_th = __builtin_fmaf(th[k], th[k], s_th);
        s_u = __builtin_fmaf(u, u, s_u);
        m[k] = m_k; v[k] = v_k;
      }
      st<NT>(m4 + i, f32_to_mom<MomV>(m));
      st<NT>(v4 + i, v);
    }
    done = nvec << 2;
  }
  for (int i = done + threadIdx.x; i < n; i += kScaledBlock) {
    const float th = th_p[i];
    float m = load_mom<MomS>(m_p + i), v = v_p[i], g, m_hat;
    if constexpr (sizeof(GradS) == 2) g = bf16_to_f32(g_p[i]);
    else g = g_p[i];
    s_g = __builtin_fmaf(g, g, s_g);
    if (gi.cols) g = centralize_one(g, off + i, gi);
    moments<AB>(th, g, m, v, c, gs);
    m = round_mom<MomS>(m);
    const float u = direction(m, v, c, m_hat);
    s_th = __builtin_fmaf(th, th, s_th);
    s_u = __builtin_fmaf(u, u, s_u);
    store_mom<MomS>(m_p + i, m);
    v_p[i] = v;
  }
  s_th = wave_sum(s_th);
  s_u = wave_sum(s_u);
  s_g = wave_sum(s_g);
  if (threadIdx.x == 0) {
    NormPartial p;
    p.theta2 = s_th; p.u2 = s_u; p.g2 = s_g; p.pad = 0.0f;
    partials[blockIdx.x] = p;
  }
}

template <typename GradS, typename GradV, bool NT, typename MomS, typename MomV, bool AB>
__global__ __launch_bounds__(kScaledBlock) void novak_moments_kernel(Tables tb, Consts c, int sub_shift, NormPartial *partials) {
  moments_body<GradS, GradV, NT, MomS, MomV, false, AB>(tb, c, sub_shift, partials, nullptr);
}
template <typename GradS, typename GradV, bool NT, typename MomS, typename MomV, bool AB>
__global__ __launch_bounds__(kScaledBlock) void novak_moments_device_kernel(Tables tb, const DeviceStep *ds, int sub_shift, NormPartial *partials) {
  moments_body<GradS, GradV, NT, MomS, MomV, true, AB>(tb, Consts(), sub_shift, partials, ds);
}

// one wave per chunk: sums the chunk's per-wave partials in a fixed order
__global__ __launch_bounds__(64) void novak_reduce_chunks_kernel(const novak_chunk *chunks, int sub_shift, int sub_elems,
                                                                 const NormPartial *partials, NormSums *chunk_sums) {
  const novak_chunk ch = chunks[blockIdx.x];
  const int nsub = (ch.len + sub_elems - 1) / sub_elems;
  const NormPartial *p = partials + (static_cast<size_t>(blockIdx.x) << sub_shift);
  double a = 0.0, b = 0.0, g = 0.0;
  for (int j = threadIdx.x; j < nsub; j += 64) {
    const NormPartial x = p[j];
    a += static_cast<double>(x.theta2);
    b += static_cast<double>(x.u2);
    g += static_cast<double>(x.g2);
  }
  a = wave_sum(a); b = wave_sum(b); g = wave_sum(g);
  if (threadIdx.x == 0) {
    NormSums s; s.theta2 = a; s.u2 = b; s.g2 = g;
    chunk_sums[blockIdx.x] = s;
  }
}

// Gradient pre-pass (Phase 2): ONE read of the gradients serves both consumers that need a whole-array
// statistic before any element may be updated - the global norm of gradient clipping (sections 5.8, 7.3)
// and the row means of gradient centralization (Eq. 26).
//   * A wave takes one chunk-table entry in spans of kPreSub = 4096 consecutive elements, 16 independent
//     128-bit loads per lane in flight: a read-only stream needs about 100 KB outstanding per compute unit,
//     and 16 KB per wave at a residency of 6 waves measured best on MI355X (7.35 TB/s against 6.8 TB/s for
//     4 KB per wave).  The next span's loads are issued before the current span is reduced.
//   * NORM: every lane keeps four fp32 sums of squares across spans; once per four spans (a chunk of the default
//     size) they are added up over the wave and into the chunk's sum (double), which the wave writes itself; the
//     tensor reduction is shared with the two-pass step, then novak_clip_kernel turns the norm into the factor
//     min(1, c_clip/||g||).
//   * GC: every row piece that lies in a span is summed in double and in a fixed order - in registers when
//     rows are made of whole 256-element pieces, else from a copy of the span parked in LDS.  Rows that lie entirely inside the span get their mean written here; a row
//     that sticks out at the front ("head") or at the back ("tail") leaves a partial sum, and
//     novak_rowfinal_kernel adds those up in wave order.  Nothing depends on timing.
constexpr int kPreUnroll = 16;
constexpr int kPreSub = kScaledSub * kPreUnroll;        // elements per wave
constexpr unsigned kPreStageBytes = kPreSub * sizeof(float);

struct RowPartial {   // per pre-pass span: the pieces of the (at most two) rows that stick out of its span
  double head, tail;
};

// Wave-wide sums through the data-parallel-primitive lane shifts instead of LDS permutes: an inclusive scan
// inside each row of 16 lanes (shift right by 1, 2, 4, 8; lanes without a source add 0), then lane 15 of
// rows 0 and 2 is added into rows 1 and 3, then lane 31 into rows 2 and 3.  The TOTAL ENDS UP IN LANE 63
// ONLY.  About four times shorter than six permute rounds, which matters to a kernel whose waves are few
// and end with this reduction.  The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_take(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_take(double x) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, ROW_MASK, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <typename T>
__device__ __forceinline__ T wave_total_in_lane63(T x) {
  x += dpp_take<0x111, 0xf>(x);    // row_shr:1
  x += dpp_take<0x112, 0xf>(x);    // row_shr:2
  x += dpp_take<0x114, 0xf>(x);    // row_shr:4
  x += dpp_take<0x118, 0xf>(x);    // row_shr:8
  x += dpp_take<0x142, 0xa>(x);    // row_bcast:15 into rows 1 and 3
  x += dpp_take<0x143, 0xc>(x);    // row_bcast:31 into rows 2 and 3
  return x;
}

// Sum of stage[a, b) over the wave, in double, fixed order: lanes take a strided share, then the scan above.
__device__ __forceinline__ double stage_sum_wave(const float *stage, int a, int b) {
  double acc = 0.0;
  if (((a | b) & 3) == 0) {
    for (int i = a + 4 * static_cast<int>(threadIdx.x); i < b; i += 256) {
      const f32x4 x = *reinterpret_cast<const f32x4 *>(stage + i);
      acc += (static_cast<double>(x[0]) + x[1]) + (static_cast<double>(x[2]) + x[3]);
    }
  } else {
    for (int i = a + static_cast<int>(threadIdx.x); i < b; i += 64) acc += static_cast<double>(stage[i]);
  }
  return wave_total_in_lane63(acc);
}

// Where the sum of one row piece goes: a row that lies entirely in the span [off, end) gets its mean, a row
// that begins before the span leaves a head piece, one that runs past its end a tail piece.
__device__ __forceinline__ void emit_row(double sum, int64_t r, int64_t cols, double inv_cols, int64_t off, int64_t end, double *means,
                                         RowPartial *rp) {
  const int64_t lo = r * cols, hi = lo + cols;
  if (lo >= off && hi <= end) means[r] = sum * inv_cols;      // a double division here costs the wave ~200 cycles per row
  else if (lo < off) rp->head = sum;
  else rp->tail = sum;
}

// What the spans of one chunk share.
template <typename GradS>
struct PreChunk {
  const GradS *g;          // the chunk's first gradient element
  int64_t offset;          // its element offset inside the tensor
  int len;
  bool gc;                 // this tensor is centralized
  GcInfo gi;
  RowPartial *row_partials;
};

// The lanes' sums of squares (four fp32 accumulators each, kept across spans) are added up over the wave once per
// kFlushSpans spans, i.e. once per chunk of the default size: 64 squares per accumulator between two flushes.  The
// spans of a chunk are taken in order by one wave, so the chunk's sum has a fixed order of additions.  (Total
// meaningful in lane 63 only.)
constexpr int kFlushSpans = 4;
template <bool NORM>
__device__ __forceinline__ void flush_norm(float (&s_g)[4], double &chunk_g2) {
  if (!NORM) return;
  chunk_g2 += static_cast<double>(wave_total_in_lane63((s_g[0] + s_g[1]) + (s_g[2] + s_g[3])));
  s_g[0] = s_g[1] = s_g[2] = s_g[3] = 0.0f;
}

// Row sums of a span whose n elements are parked in LDS.
__device__ __forceinline__ void rows_from_stage(const float *stage, int64_t off, int n, const GcInfo &gi, RowPartial *rp) {
  __syncthreads();                                      // one wave: orders the LDS writes before the reads
  const int64_t cols = gi.cols, end = off + n;
  double *means = const_cast<double *>(gi.means);
  const int64_t r_first = row_of(off, cols, gi.inv_cols), r_last = row_of(end - 1, cols, gi.inv_cols);
  if (r_last - r_first >= 64) {
    // many short rows: one lane per row, elements summed in order
    for (int64_t r = r_first + threadIdx.x; r <= r_last; r += kScaledBlock) {
      const int64_t lo = r * cols, hi = lo + cols;
      const int a = static_cast<int>((lo > off ? lo : off) - off), b = static_cast<int>((hi < end ? hi : end) - off);
      double acc = 0.0;
      for (int i = a; i < b; ++i) acc += static_cast<double>(stage[i]);
      emit_row(acc, r, cols, gi.inv_cols, off, end, means, rp);
    }
  } else {
    // few long rows: the whole wave sums one row piece after the other
    for (int64_t r = r_first; r <= r_last; ++r) {
      const int64_t lo = r * cols, hi = lo + cols;
      const int a = static_cast<int>((lo > off ? lo : off) - off), b = static_cast<int>((hi < end ? hi : end) - off);
      const double sum = stage_sum_wave(stage, a, b);
      if (threadIdx.x == 63) emit_row(sum, r, cols, gi.inv_cols, off, end, means, rp);
    }
  }
  __syncthreads();                                      // the next span of this wave reuses the buffer
}

// A full, aligned span whose 16 vectors per lane are already in registers.  (Norm first, row sums in a second
// sweep: one merged sweep measured 1-13 % slower, the scans between the pieces hold up the arriving loads.)
template <typename GradS, typename GradV, bool NORM>
__device__ __forceinline__ void span_from_registers(const GradV (&g)[kPreUnroll], int s, const PreChunk<GradS> &pc, float *stage, float (&s_g)[4]) {
  const int64_t off = pc.offset + static_cast<int64_t>(s) * kPreSub, end = off + kPreSub;
  if (NORM) {
#pragma unroll
    for (int u = 0; u < kPreUnroll; ++u) {
      const f32x4 gf = grad_to_f32<GradV>(g[u]);
#pragma unroll
      for (int k = 0; k < 4; ++k) s_g[u & 3] = __builtin_fmaf(gf[k], gf[k], s_g[u & 3]);
    }
  }
  if (!pc.gc) return;
  const int64_t cols = pc.gi.cols;
  RowPartial *rp = pc.row_partials + s;
  if ((cols & 255) == 0) {
    // Rows made of whole 256-element pieces: piece u is what the wave's u-th load fetched and lies inside one
    // row, so the row sums form in registers - lanes add their vectors over a row's pieces, then one scan per
    // row.  Every branch is uniform.
    double *means = const_cast<double *>(pc.gi.means);
    int64_t r = row_of(off, cols, pc.gi.inv_cols);
    int left = static_cast<int>((r * cols + cols - off) >> 8);     // pieces of row r from the span's start on
    double acc = 0.0;
#pragma unroll
    for (int u = 0; u < kPreUnroll; ++u) {
      const f32x4 gf = grad_to_f32<GradV>(g[u]);
      acc += (static_cast<double>(gf[0]) + gf[1]) + (static_cast<double>(gf[2]) + gf[3]);
      if (--left == 0 || u == kPreUnroll - 1) {
        const double sum = wave_total_in_lane63(acc);
        if (threadIdx.x == 63) emit_row(sum, r, cols, pc.gi.inv_cols, off, end, means, rp);
        ++r;
        left = static_cast<int>(cols >> 8);
        acc = 0.0;
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < kPreUnroll; ++u)
      *reinterpret_cast<f32x4 *>(stage + 4 * (threadIdx.x + u * kScaledBlock)) = grad_to_f32<GradV>(g[u]);
    rows_from_stage(stage, off, kPreSub, pc.gi, rp);
  }
}

// Any other span (the ragged last one of a tensor, or a gradient that is not 16-byte aligned): loads as it goes.
template <typename GradS, typename GradV, bool NT, bool NORM>
__device__ __forceinline__ void span_generic(int s, const PreChunk<GradS> &pc, float *stage, float (&s_g)[4]) {
  const int start = s * kPreSub;
  const int n = min(kPreSub, pc.len - start);
  const GradS *__restrict__ g_p = pc.g + start;
  int done = 0;
  if ((reinterpret_cast<uintptr_t>(g_p) & (sizeof(GradV) - 1)) == 0) {
    const GradV *g4 = reinterpret_cast<const GradV *>(g_p);
    const int nvec = n >> 2;
    for (int i = threadIdx.x; i < nvec; i += kScaledBlock) {
      const f32x4 gf = grad_to_f32<GradV>(ld<NT>(g4 + i));
      if (NORM) {
#pragma unroll
        for (int k = 0; k < 4; ++k) s_g[k] = __builtin_fmaf(gf[k], gf[k], s_g[k]);
      }
      if (pc.gc) *reinterpret_cast<f32x4 *>(stage + 4 * i) = gf;
    }
    done = nvec << 2;
  }
  for (int i = done + threadIdx.x; i < n; i += kScaledBlock) {
    float g;
    if constexpr (sizeof(GradS) == 2) g = bf16_to_f32(g_p[i]);
    else g = g_p[i];
    if (NORM) s_g[0] = __builtin_fmaf(g, g, s_g[0]);
    if (pc.gc) stage[i] = g;
  }
  if (pc.gc) rows_from_stage(stage, pc.offset + start, n, pc.gi, pc.row_partials + s);
}

// One wave per chunk-table entry.  The chunk's spans are taken in order, and the loads of the next full span
// are issued before the current one is reduced, so the wave's memory pipe does not idle while it adds up.
template <typename GradS, typename GradV, bool NT, bool NORM, bool GC>
__global__ __launch_bounds__(kScaledBlock) void novak_prepass_kernel(Tables tb, int sub_shift, NormSums *chunk_sums,
                                                                     RowPartial *row_partials) {
  extern __shared__ __align__(16) float stage[];                      // kPreSub floats, touched only on the staged centralization path
  const novak_chunk ch = tb.chunks[blockIdx.x];
  PreChunk<GradS> pc;
  pc.g = static_cast<const GradS *>(tb.grad[ch.tensor]) + ch.offset;
  pc.offset = ch.offset;
  pc.len = ch.len;
  pc.gi.cols = 0;
  if (GC) pc.gi = tb.gc[ch.tensor];
  pc.gc = GC && pc.gi.cols > 0;
  double chunk_g2 = 0.0;
  float s_g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  pc.row_partials = row_partials + (static_cast<size_t>(blockIdx.x) << sub_shift);
  const int nspans = (ch.len + kPreSub - 1) / kPreSub;
  const int nfull = (reinterpret_cast<uintptr_t>(pc.g) & (sizeof(GradV) - 1)) == 0 ? ch.len / kPreSub : 0;
  const GradV *g4 = reinterpret_cast<const GradV *>(pc.g) + threadIdx.x;
  constexpr int kSpanVecs = kPreSub / 4;
  GradV a[kPreUnroll], b[kPreUnroll];
  if (nfull > 0) {
#pragma unroll
    for (int u = 0; u < kPreUnroll; ++u) a[u] = ld<NT>(g4 + u * kScaledBlock);
  }
  for (int s = 0; s < nspans; s += 2) {
    if (s + 1 < nfull) {
#pragma unroll
      for (int u = 0; u < kPreUnroll; ++u) b[u] = ld<NT>(g4 + (s + 1) * kSpanVecs + u * kScaledBlock);
    }
    if (s < nfull) span_from_registers<GradS, GradV, NORM>(a, s, pc, stage, s_g);
    else span_generic<GradS, GradV, NT, NORM>(s, pc, stage, s_g);
    if (s + 1 >= nspans) break;
    if (s + 2 < nfull) {
#pragma unroll
      for (int u = 0; u < kPreUnroll; ++u) a[u] = ld<NT>(g4 + (s + 2) * kSpanVecs + u * kScaledBlock);
    }
    if (s + 1 < nfull) span_from_registers<GradS, GradV, NORM>(b, s + 1, pc, stage, s_g);
    else span_generic<GradS, GradV, NT, NORM>(s + 1, pc, stage, s_g);
    if (((s + 2) & (kFlushSpans - 1)) == 0) flush_norm<NORM>(s_g, chunk_g2);
  }
  flush_norm<NORM>(s_g, chunk_g2);
  if (NORM && threadIdx.x == 63) {
    NormSums sums;
    sums.theta2 = 0.0; sums.u2 = 0.0; sums.g2 = chunk_g2;
    chunk_sums[blockIdx.x] = sums;
  }
}

// Means of the rows whose elements are spread over several pre-pass waves: the first wave's tail piece,
// then the head pieces of the following waves, in order.  One lane per row of the centralized tensors;
// `gc_tensor[j]` lists them, `row_first[j]` is the index of tensor j's first row (prefix sums, n_gc + 1
// entries), `first_chunk[t]` the tensor's first chunk-table entry.
__global__ __launch_bounds__(64) void novak_rowfinal_kernel(const int *gc_tensor, const int64_t *row_first, int n_gc, const GcInfo *gc,
                                                           const int *first_chunk, int sub_shift, int64_t total_rows,
                                                           const RowPartial *row_partials, double *means) {
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 64 + threadIdx.x;
  if (row >= total_rows) return;
  int lo = 0, hi = n_gc - 1;                     // largest j with row_first[j] <= row
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (row_first[mid] <= row) lo = mid;
    else hi = mid - 1;
  }
  const int t = gc_tensor[lo];
  const int64_t r = row - row_first[lo];
  const int64_t cols = gc[t].cols;
  const int64_t w_a = (r * cols) / kPreSub, w_b = (r * cols + cols - 1) / kPreSub;   // pre-pass waves of this tensor
  if (w_a == w_b) return;                        // the row lies inside one wave's span: its mean is already there
  const RowPartial *p = row_partials + (static_cast<int64_t>(first_chunk[t]) << sub_shift);
  double sum = p[w_a].tail;
  for (int64_t w = w_a + 1; w <= w_b; ++w) sum += p[w].head;
  means[row] = sum * gc[t].inv_cols;
}

__global__ __launch_bounds__(64) void novak_clip_kernel(int n_tensors, const NormSums *tensor_sums, float c_clip, float *gscale) {
  double g = 0.0;
  for (int j = threadIdx.x; j < n_tensors; j += 64) g += tensor_sums[j].g2;
  g = wave_sum(g);
  if (threadIdx.x == 0) {
    const double norm = sqrt(g);
    gscale[0] = norm > static_cast<double>(c_clip) ? static_cast<float>(static_cast<double>(c_clip) / norm) : 1.0f;
  }
}

struct ScaleParams {
  float trust_lo, trust_hi;    // clip range of Eq. 19
  float auto_lo, auto_hi;      // clip range of Eq. 22
  double gamma;                // EMA weight of Eq. 20-21
  int layer_adaptation, auto_lr;
};

// one workgroup of eight waves per tensor: per-tensor sums in a fixed order (lanes take a strided share of the
// tensor's chunk sums, a tree per wave, then the waves in order); the clipped trust ratio (Eq. 19 / 25) goes to
// scale[t].  (One wave per tensor took 28 us on a tensor of 6000 chunks, between the two passes of every step.)
constexpr int kTensorReduceBlock = 512;
__global__ __launch_bounds__(kTensorReduceBlock) void novak_reduce_tensors_kernel(const int *first_chunk, const NormSums *chunk_sums,
                                                                                  NormSums *tensor_sums, float *scale, ScaleParams sp) {
  __shared__ double part[kTensorReduceBlock / 64][3];
  const int t = blockIdx.x;
  const int c0 = first_chunk[t], c1 = first_chunk[t + 1];
  double a = 0.0, b = 0.0, g = 0.0;
  for (int j = c0 + threadIdx.x; j < c1; j += kTensorReduceBlock) {
    const NormSums x = chunk_sums[j];
    a += x.theta2; b += x.u2; g += x.g2;
  }
  a = wave_sum(a); b = wave_sum(b); g = wave_sum(g);
  if ((threadIdx.x & 63) == 0) {
    part[threadIdx.x >> 6][0] = a; part[threadIdx.x >> 6][1] = b; part[threadIdx.x >> 6][2] = g;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = b = g = 0.0;
    for (int w = 0; w < kTensorReduceBlock / 64; ++w) { a += part[w][0]; b += part[w][1]; g += part[w][2]; }
    NormSums s; s.theta2 = a; s.u2 = b; s.g2 = g;
    tensor_sums[t] = s;
    float eta = 1.0f;
    if (sp.layer_adaptation) {
      // eta = ||theta|| / ||u||, 1 when either norm is zero; clipped
      double r = (a > 0.0 && b > 0.0) ? sqrt(a / b) : 1.0;
      r = r < static_cast<double>(sp.trust_lo) ? static_cast<double>(sp.trust_lo) : r;
      r = r > static_cast<double>(sp.trust_hi) ? static_cast<double>(sp.trust_hi) : r;
      eta = static_cast<float>(r);
    }
    scale[t] = eta;
  }
}

// one wave: global norms -> EMAs (Eq. 20-21, state in `ema`: g_bar, theta_bar) -> alpha_auto (Eq. 22),
// folded into every tensor's scale.  `theta_sums` (when given): the parameters' sums of squares come from a pre-pass of
// their own, in its g2 field; `ascale` (when given) receives alpha_auto for the single-pass step.
__global__ __launch_bounds__(64) void novak_auto_lr_kernel(int n_tensors, const NormSums *tensor_sums, float *scale,
                                                           double *ema, ScaleParams sp, const NormSums *theta_sums, float *ascale) {
  double a = 0.0, g = 0.0;
  for (int j = threadIdx.x; j < n_tensors; j += 64) {
    a += theta_sums ? theta_sums[j].g2 : tensor_sums[j].theta2;
    g += tensor_sums[j].g2;
  }
  a = wave_sum(a); g = wave_sum(g);
  // every lane holds the same sums; every lane computes the same factor
  const double g_bar = sp.gamma * sqrt(g) + (1.0 - sp.gamma) * ema[0];
  const double th_bar = sp.gamma * sqrt(a) + (1.0 - sp.gamma) * ema[1];
  double f = 1.0;
  if (th_bar != 0.0) {
    f = g_bar / th_bar;
    f = f < static_cast<double>(sp.auto_lo) ? static_cast<double>(sp.auto_lo) : f;
    f = f > static_cast<double>(sp.auto_hi) ? static_cast<double>(sp.auto_hi) : f;
  }
  const float ff = static_cast<float>(f);
  for (int j = threadIdx.x; j < n_tensors; j += 64) scale[j] *= ff;
  __syncthreads();   // all lanes have read ema before lane 0 replaces it
  if (threadIdx.x == 0) {
    ema[0] = g_bar;
    ema[1] = th_bar;
    if (ascale) *ascale = ff;
  }
}

// LA is a phase, or (device-step mode) LA_RUNTIME_ME / LA_RUNTIME_BASIC with the phase in `ds`, as in step_body.
template <int LA, bool NT, typename MomS, typename MomV, bool DEV>
__device__ __forceinline__ void apply_body(const Tables &tb, const Consts &c_arg, int sub_shift, const float *scale, const DeviceStep *ds) {
  const novak_chunk ch = tb.chunks[blockIdx.x >> sub_shift];
  const int start = static_cast<int>(blockIdx.x & ((1u << sub_shift) - 1u)) * kScaledSub;
  if (start >= ch.len) return;
  const int n = min(kScaledSub, ch.len - start);
  const int64_t off = ch.offset + start;
  const TensorPtrs tp = tb.tensors[ch.tensor];
  DeviceStep d;
  if constexpr (DEV) d = *ds;
  const Consts &c = DEV ? d.c : c_arg;
  const int la_rt = DEV ? d.la : LA_OFF;
  const int phase = la_runtime(LA) ? la_rt : LA;
  const bool reads = la_reads(phase), writes = la_writes(phase);
  const float step = c.step_size * scale[ch.tensor];                    // Eq. 24a
  if constexpr (DEV) device_step_done(d);      // (after the wave-uniform loads: see step_body)
  float *__restrict__ th_p = tp.param + off;
  const MomS *__restrict__ m_p = reinterpret_cast<const MomS *>(tp.m) + off;
  const float *__restrict__ v_p = tp.v + off;
  float *__restrict__ la_p = nullptr;
  if (LA != LA_OFF) la_p = tp.la + off;
  const uintptr_t mis = ((reinterpret_cast<uintptr_t>(th_p) | reinterpret_cast<uintptr_t>(v_p) | reinterpret_cast<uintptr_t>(la_p)) & 15u) |
                        (reinterpret_cast<uintptr_t>(m_p) & (sizeof(MomV) - 1));
  int done = 0;
  if (mis == 0) {
    const int nvec = n >> 2;
    f32x4 *th4 = reinterpret_cast<f32x4 *>(th_p);
    const MomV *m4 = reinterpret_cast<const MomV *>(m_p);
    const f32x4 *v4 = reinterpret_cast<const f32x4 *>(v_p);
    f32x4 *la4 = reinterpret_cast<f32x4 *>(la_p);
    const int i = threadIdx.x;
    if (i < nvec) {
      // (run-time phase: the lookahead load is issued whatever the phase, from theta's address when unused - see step_body)
      const f32x4 *la_src = (la_runtime(LA) && !reads) ? th4 : la4;
      f32x4 th = ld<NT>(th4 + i), la = {0.0f, 0.0f, 0.0f, 0.0f};
      const f32x4 m = mom_to_f32<MomV>(ld<NT>(m4 + i)), v = ld<NT>(v4 + i);
      if (la_runtime(LA) || reads) la = ld<NT>(la_src + i);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float th_k = th[k], la_k = la[k], m_hat;
        const float u = direction(m[k], v[k], c, m_hat);
        apply<LA>(th_k, u, m_hat, la_k, c, step, la_rt);
        th[k] = th_k; la[k] = la_k;
      }
      st<NT>(th4 + i, th);
      if (writes) st<NT>(la4 + i, la);
    }
    done = nvec << 2;
  }
  for (int i = done + threadIdx.x; i < n; i += kScaledBlock) {
    float th = th_p[i], la = 0.0f, m_hat;
    if (reads) la = la_p[i];
    const float u = direction(load_mom<MomS>(m_p + i), v_p[i], c, m_hat);
    apply<LA>(th, u, m_hat, la, c, step, la_rt);
    th_p[i] = th;
    if (writes) la_p[i] = la;
  }
}

template <int LA, bool NT, typename MomS = float, typename MomV = f32x4>
__global__ __launch_bounds__(kScaledBlock) void novak_apply_kernel(Tables tb, Consts c, int sub_shift, const float *scale) {
  apply_body<LA, NT, MomS, MomV, false>(tb, c, sub_shift, scale, nullptr);
}
template <int LA, bool NT, typename MomS = float, typename MomV = f32x4>
__global__ __launch_bounds__(kScaledBlock) void novak_apply_device_kernel(Tables tb, const DeviceStep *ds, int sub_shift, const float *scale) {
  apply_body<LA, NT, MomS, MomV, true>(tb, Consts(), sub_shift, scale, ds);
}

// ------------------------------------------------------------------------------------------------
// Tables of the allocation-free step, written on the device from kernel arguments (no host-to-device
// copy, which could allocate staging memory): one workgroup per tensor of the batch writes the
// tensor's pointer record, its gradient pointer, its chunk range and its chunk-table entries.
// ------------------------------------------------------------------------------------------------
constexpr int kFillBatch = 64;   // tensors per launch: 64 x 56 bytes of arguments stay below the 4 KB limit

struct FillTensor {
  TensorPtrs ptrs;
  const void *grad;
  int64_t numel;
  int64_t first_chunk;           // index of the tensor's first chunk-table entry
};
struct FillBatch {
  int32_t count;                 // tensors in this batch
  int32_t first_tensor;          // index of the batch's first tensor in the list
  int32_t n_tensors;             // tensors in the whole list
  int32_t n_chunks;              // chunk-table entries of the whole list
  int64_t chunk_elems;
  FillTensor t[kFillBatch];
};

__global__ __launch_bounds__(64) void novak_fill_tables_kernel(FillBatch b, novak_chunk *chunks, TensorPtrs *tensors,
                                                              const void **grad, int *first_chunk) {
  const int j = blockIdx.x;
  if (j >= b.count) return;
  const FillTensor &ft = b.t[j];
  const int t = b.first_tensor + j;
  if (threadIdx.x == 0) {
    tensors[t] = ft.ptrs;
    grad[t] = ft.grad;
    first_chunk[t] = static_cast<int>(ft.first_chunk);
    if (t == b.n_tensors - 1) first_chunk[b.n_tensors] = b.n_chunks;
  }
  const int64_t n = (ft.numel + b.chunk_elems - 1) / b.chunk_elems;
  for (int64_t k = threadIdx.x; k < n; k += 64) {
    novak_chunk c;
    c.offset = k * b.chunk_elems;
    c.tensor = t;
    const int64_t rest = ft.numel - c.offset;
    c.len = static_cast<int32_t>(rest < b.chunk_elems ? rest : b.chunk_elems);
    chunks[ft.first_chunk + k] = c;
  }
}

}  // namespace

#endif  // NOVAK_KERNELS_H_
