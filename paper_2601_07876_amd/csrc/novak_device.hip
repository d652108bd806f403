// Host side of the device part of the NOVAK update-step library: the handle, launch geometry and
// the C entry points that enqueue the kernels of novak_kernels.h on the caller's HIP stream.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "novak_internal.h"
#include "novak_kernels.h"

namespace {
thread_local std::string g_create_error = "";
}  // namespace

// ------------------------------------------------------------------------------------------------
// Static scratch of the allocation-free step (novak_step_static): chunk table, pointer records,
// gradient pointers and the clipping pre-pass's reduction buffers live here instead of in hipMalloc'ed
// memory.  Every GPU the library runs on holds its own copy of the array until the process ends; host
// code reaches it only through the address hipGetSymbolAddress returns for the current device.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[NOVAK_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};   // per device, filled on the first call on that device

// Device address of `scratch` on device `dev`, which must be the current device.
hipError_t scratch_of(int dev, unsigned char **out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

// Everything a kernel launch needs: effective hyper-parameters, geometry, tuning and the device-side
// tables.  A handle owns one whose tables come from hipMalloc; the allocation-free entry point builds one
// over the library's static scratch array.
struct LaunchCtx {
  novak_hparams hp;                 // effective hyper-parameters
  int32_t n_tensors = 0;
  int64_t chunk_elems = NOVAK_CHUNK_DEFAULT;
  int64_t n_chunks = 0;
  int nontemporal = 1;
  int vec_per_lane = 1;             // 128-bit accesses per stream per lane (UN): 1, 2 or 4
  int threads = 64;                 // workgroup size: 64, 128 or 256 (one to four wave64)
  int waves_per_cu = 0;             // cap on resident waves per compute unit; 0 = chosen per kernel variant
  int prepass_waves_per_cu = 0;     // the same for the gradient pre-pass
  int lds_per_cu = 160 * 1024;      // LDS of one compute unit (queried at create)
  // reduction scratch of the two-pass path (layer adaptation / auto-LR) and of the clipping pre-pass
  NormPartial *d_partials = nullptr;   // one per wave of pass 1
  NormSums *d_chunk_sums = nullptr;    // one per chunk
  NormSums *d_tensor_sums = nullptr;   // one per tensor
  int *d_first_chunk = nullptr;        // n_tensors + 1: chunk range of each tensor
  float *d_scale = nullptr;            // n_tensors: lambda_trust * alpha_auto
  float *d_gscale = nullptr;           // one float: gradient-clipping factor of the current step
  // auto-LR without a trust ratio: global norms from pre-passes, the factor of Eq. 22 in one float
  float *d_ascale = nullptr;
  NormSums *d_chunk_sums_theta = nullptr;   // one per chunk: sums of squares of the parameters (in the g2 field)
  NormSums *d_tensor_sums_theta = nullptr;  // one per tensor
  const void **d_theta_ptrs = nullptr;      // n_tensors parameter pointers, for the pre-pass over theta
  // gradient centralization
  GcInfo *d_gc = nullptr;              // per tensor
  int *d_gc_tensor = nullptr;          // centralized tensors
  int64_t *d_row_first = nullptr;      // their first rows (prefix sums, n_gc + 1)
  double *d_row_means = nullptr;       // one double per row
  RowPartial *d_row_partials = nullptr;   // one per pre-pass wave (rebuilt with the chunk table)
  int n_gc = 0;
  int64_t total_rows = 0;
  double *d_ema = nullptr;             // caller-owned: g_bar, theta_bar
  // device-step mode
  DeviceStep *d_step = nullptr;        // the record of the step being enqueued (a slot of the handle's ring of kDeviceRing)
  int64_t *d_counter = nullptr;        // caller-owned: steps taken so far
  // tables
  novak_chunk *d_chunks = nullptr;
  void *d_ptrs = nullptr;           // n_tensors TensorPtrs records, then n_tensors gradient pointers
};

// ------------------------------------------------------------------------------------------------
// handle
// ------------------------------------------------------------------------------------------------
struct novak_handle : LaunchCtx {
  uint32_t warnings = 0;
  int32_t device_id = 0;
  std::vector<novak_tensor_desc> tensors;
  std::vector<int64_t> numels;
  int64_t total_numel = 0;
  int64_t last_step = 0;
  int sync_due = 0;
  float **d_out_ptrs = nullptr;        // n_tensors output pointers of novak_nesterov_extrapolate (allocated in create)
  // pinned staging ring for the per-step gradient pointer list
  static constexpr int kRing = 4;
  void **h_ring = nullptr;
  hipEvent_t ring_ev[kRing] = {};
  bool ring_used[kRing] = {};
  int ring_next = 0;
  std::vector<void *> last_grads;
  // one more pinned slot (index kRing of h_ring) stages novak_nesterov_extrapolate's pointer list
  hipEvent_t out_ev = nullptr;
  bool out_used = false;
  bool grads_uploaded = false;
  // device-step mode: the ring of step records.  Eagerly every step has its record written just before it (slot 0);
  // under stream capture one prologue writes kDeviceRing records ahead and the captured steps take consecutive slots,
  // so a replayed graph is self-contained: it starts by reading the counter and needs no further prologue.
  DeviceStep *d_ring = nullptr;
  int dev_slot = 0;                          // next slot of the capture in progress
  unsigned long long dev_capture_id = 0;     // which capture the slots belong to
  bool dev_in_capture = false;
  bool broken = false;              // a table rebuild failed half way: every later call is refused
  std::string error;
};

namespace {

int fail(novak_handle *h, int status, const std::string &msg) {
  if (h) h->error = msg;
  else g_create_error = msg;
  return status;
}

int fail_hip(novak_handle *h, hipError_t e, const char *what) {
  return fail(h, NOVAK_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define NOVAK_HIP(h, call)                                   \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return fail_hip((h), e_, #call);   \
  } while (0)

// RAII: make the handle's device current for the duration of a call, then restore.
struct DeviceScope {
  int prev = -1;
  bool switched = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      if (e != hipSuccess) return e;
      switched = true;
    }
    return hipSuccess;
  }
  ~DeviceScope() {
    if (switched) (void)hipSetDevice(prev);
  }
};

Tables tables_of(const LaunchCtx *h) {
  const size_t n = static_cast<size_t>(h->n_tensors);
  char *base = static_cast<char *>(h->d_ptrs);
  Tables tb;
  tb.chunks = h->d_chunks;
  tb.tensors = reinterpret_cast<const TensorPtrs *>(base);
  tb.grad = reinterpret_cast<const void *const *>(base + n * sizeof(TensorPtrs));
  tb.gscale = h->d_gscale;
  tb.gc = h->d_gc;
  tb.ascale = h->d_ascale;
  return tb;
}

// The trust ratio needs per-tensor norms of the direction: two passes.  Auto-LR alone needs the global norms of the
// gradients and the parameters as they are before the step: a pre-pass over each, then the single-pass step.
bool two_pass(const LaunchCtx *h) { return h->hp.layer_adaptation != 0; }
bool auto_only(const LaunchCtx *h) { return h->hp.auto_lr && !h->hp.layer_adaptation; }
bool scaled(const LaunchCtx *h) { return h->hp.layer_adaptation || h->hp.auto_lr; }
bool clipping(const LaunchCtx *h) { return h->hp.clip_threshold > 0.0; }
bool needs_reductions(const LaunchCtx *h) { return scaled(h) || clipping(h); }

void free_device_tables(novak_handle *h) {
  if (h->d_chunks) (void)hipFree(h->d_chunks);
  if (h->d_partials) (void)hipFree(h->d_partials);
  if (h->d_chunk_sums) (void)hipFree(h->d_chunk_sums);
  if (h->d_tensor_sums) (void)hipFree(h->d_tensor_sums);
  if (h->d_first_chunk) (void)hipFree(h->d_first_chunk);
  if (h->d_scale) (void)hipFree(h->d_scale);
  if (h->d_gscale) (void)hipFree(h->d_gscale);
  if (h->d_ascale) (void)hipFree(h->d_ascale);
  if (h->d_chunk_sums_theta) (void)hipFree(h->d_chunk_sums_theta);
  if (h->d_tensor_sums_theta) (void)hipFree(h->d_tensor_sums_theta);
  h->d_ascale = nullptr;
  h->d_chunk_sums_theta = nullptr;
  h->d_tensor_sums_theta = nullptr;
  if (h->d_row_partials) (void)hipFree(h->d_row_partials);
  h->d_row_partials = nullptr;
  h->d_gscale = nullptr;
  h->d_chunks = nullptr;
  h->d_partials = nullptr;
  h->d_chunk_sums = nullptr;
  h->d_tensor_sums = nullptr;
  h->d_first_chunk = nullptr;
  h->d_scale = nullptr;
}

int build_chunk_table_unguarded(novak_handle *h);
bool fits_one_launch(int64_t n_chunks, int64_t chunk_elems);
constexpr const char *kTooLarge = "the tensor list needs more than 2^32 - 1 threads in one launch (about 1.7e10 elements); split it over several handles";

// (Re)build and upload the chunk table for the current chunk_elems.  Synchronous.  If it fails after the
// old tables were released the handle keeps no tables at all and refuses further work.
int build_chunk_table(novak_handle *h) {
  const int rc = build_chunk_table_unguarded(h);
  if (rc != NOVAK_OK && h->broken) {
    free_device_tables(h);
    h->n_chunks = 0;
  }
  return rc;
}

int build_chunk_table_unguarded(novak_handle *h) {
  int64_t n = 0;
  int rc = novak_plan_chunks(h->numels.data(), static_cast<int32_t>(h->numels.size()), h->chunk_elems, nullptr, 0, &n);
  if (rc != NOVAK_OK) return fail(h, rc, "chunk planning failed");
  if (!fits_one_launch(n, h->chunk_elems)) return fail(h, NOVAK_ERR_INVALID_ARG, kTooLarge);
  std::vector<novak_chunk> table(static_cast<size_t>(n));
  rc = novak_plan_chunks(h->numels.data(), static_cast<int32_t>(h->numels.size()), h->chunk_elems, table.data(), n, &n);
  if (rc != NOVAK_OK) return fail(h, rc, "chunk planning failed");
  free_device_tables(h);
  h->broken = true;                 // until every table below exists
  h->n_chunks = n;
  if (n > 0) {
    NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_chunks), static_cast<size_t>(n) * sizeof(novak_chunk)));
    NOVAK_HIP(h, hipMemcpy(h->d_chunks, table.data(), static_cast<size_t>(n) * sizeof(novak_chunk), hipMemcpyHostToDevice));
  }
  if ((needs_reductions(h) || h->n_gc > 0) && !h->tensors.empty()) {
    const size_t nt = h->tensors.size();
    std::vector<int> first(nt + 1, 0);
    for (const novak_chunk &c : table) first[static_cast<size_t>(c.tensor) + 1] += 1;
    for (size_t t = 0; t < nt; ++t) first[t + 1] += first[t];
    NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_first_chunk), (nt + 1) * sizeof(int)));
    NOVAK_HIP(h, hipMemcpy(h->d_first_chunk, first.data(), (nt + 1) * sizeof(int), hipMemcpyHostToDevice));
    if (h->n_gc > 0 && n > 0) {
      const size_t waves = static_cast<size_t>(n) * static_cast<size_t>(h->chunk_elems / kPreSub);
      NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_row_partials), waves * sizeof(RowPartial)));
    }
  }
  if (needs_reductions(h) && !h->tensors.empty()) {
    const size_t nt = h->tensors.size();
    const float one = 1.0f;
    NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_gscale), sizeof(float)));
    NOVAK_HIP(h, hipMemcpy(h->d_gscale, &one, sizeof(float), hipMemcpyHostToDevice));
    NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_tensor_sums), nt * sizeof(NormSums)));
    NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_scale), nt * sizeof(float)));
    std::vector<float> ones(nt, 1.0f);
    NOVAK_HIP(h, hipMemcpy(h->d_scale, ones.data(), nt * sizeof(float), hipMemcpyHostToDevice));
    if (auto_only(h)) {
      NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_ascale), sizeof(float)));
      NOVAK_HIP(h, hipMemcpy(h->d_ascale, &one, sizeof(float), hipMemcpyHostToDevice));
      NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_tensor_sums_theta), nt * sizeof(NormSums)));
      if (n > 0) NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_chunk_sums_theta), static_cast<size_t>(n) * sizeof(NormSums)));
    }
    if (n > 0) {
      NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_chunk_sums), static_cast<size_t>(n) * sizeof(NormSums)));
      if (two_pass(h)) {   // one partial per wave of pass 1 (256 elements per wave); the pre-pass writes chunk sums itself
        const size_t waves = static_cast<size_t>(n) * static_cast<size_t>(h->chunk_elems / kScaledSub);
        NOVAK_HIP(h, hipMalloc(reinterpret_cast<void **>(&h->d_partials), waves * sizeof(NormPartial)));
      }
    }
  }
  h->broken = false;
  return NOVAK_OK;
}

int log2_exact(int64_t x) {
  int s = 0;
  while ((int64_t{1} << s) < x) ++s;
  return s;
}

// grid size and sub-block shift for a kernel whose workgroups cover `sub_elems` elements each
struct Geometry {
  unsigned grid;
  int sub_shift;
  unsigned lds;   // dynamic LDS bytes requested per workgroup (never touched; bounds residency)
};
// Residency.  `wide` = arrays of 4-byte elements a wave reads plus those it writes (1 KB per wave each),
// `narrow` = the same count for 2-byte arrays (bf16 gradients, bf16 first moment; 512 bytes per wave).
// Measured on MI355X (physically contiguous arena), bandwidth peaks at 8 resident waves per compute unit
// for 9 wide arrays, 9-10 for 8, 11 for 7, 12 for 6 and 13-14 for 5, whether or not narrow arrays are
// touched as well, and falls by 5-10 % towards full occupancy: about 74 wide wave-accesses outstanding
// per compute unit.  Lists of smaller tensors (0.1-0.4 ms kernels) and the two kernels of the two-pass
// step peak one or two waves later; the budgets below are the compromise (78, and 84 for the two-pass
// kernels).  Residency is capped by requesting LDS that the kernel never touches.
constexpr double kStepBudget = 78.0, kTwoPassBudget = 84.0, kDeviceStepBudget = 99.0;
constexpr int64_t kCacheResidentElems = int64_t{1} << 22;
Geometry geometry_of(const LaunchCtx *h, int sub_elems, int threads, int wide, int narrow = 0, double budget = kStepBudget) {
  Geometry gm;
  gm.sub_shift = log2_exact(h->chunk_elems / sub_elems);
  gm.grid = static_cast<unsigned>(h->n_chunks << gm.sub_shift);
  int waves = h->waves_per_cu;                       // 0 = automatic
  if (waves == 0) {
    const double per_wave = static_cast<double>(wide > 0 ? wide : 1) * h->vec_per_lane;
    waves = static_cast<int>(budget / per_wave + 0.5);
    // with a narrow array in the mix there is no gain beyond these (the two kernels of the two-pass step with a
    // bfloat16 m plateau at 22 - 28 waves; the single-pass kernels at 14 with five wide arrays, at 16 - 18 with four)
    const int cap = budget == kTwoPassBudget ? 24 : ((budget > kStepBudget || wide <= 4) ? 16 : 14);
    if (narrow > 0 && waves > cap) waves = cap;
    // A list whose whole step fits the last-level cache (4 M elements: 150 MB) is bound by latency, not by DRAM: more waves
    // in flight are what helps there (1 M elements in a replayed graph: 6.45 -> 5.25 us per step at 16 waves; 2 M +8 %,
    // 4 M +2 %; from 8 M elements on the cap above wins by 2 - 6 %).
    if (h->n_chunks * h->chunk_elems <= kCacheResidentElems && waves < 16) waves = 16;
  }
  const int waves_per_wg = threads / 64;
  int wgs = waves / waves_per_wg;
  if (wgs < 1) wgs = 1;
  gm.lds = 0;
  if (wgs * waves_per_wg < 32) {                     // 32 waves per CU is the hardware's own limit
    unsigned bytes = (static_cast<unsigned>(h->lds_per_cu) / static_cast<unsigned>(wgs)) & ~511u;
    if (bytes > 65536u) bytes = 65536u;              // larger requests would need an opt-in attribute
    gm.lds = bytes;
  }
  return gm;
}

// arrays touched by the fused step: theta, m, v read and written, g read, the lookahead buffer per phase
struct StreamCount {
  int wide, narrow;
};
StreamCount step_streams(int grad_dtype, int la, bool bf16_m) {
  StreamCount n{4, 0};                                // theta and v, read and written
  if (bf16_m) n.narrow += 2; else n.wide += 2;        // m read and written
  if (grad_dtype == NOVAK_GRAD_BF16) n.narrow += 1; else n.wide += 1;
  if (la_reads(la)) n.wide += 1;
  if (la_writes(la)) n.wide += 1;
  return n;
}

template <typename GradS, typename GradV, bool NT, int UN, int BLOCK>
void launch_step_la(int la, const Geometry &gm, hipStream_t s, const Tables &tb, const Consts &c) {
  const dim3 grid(gm.grid), block(BLOCK);
  switch (la) {
    case LA_OFF: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_OFF, NT, UN, BLOCK>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_FIRST: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_FIRST, NT, UN, BLOCK>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_MID: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_MID, NT, UN, BLOCK>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_LAST_FUSED: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_LAST_FUSED, NT, UN, BLOCK>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    default: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_BASIC_FUSED, NT, UN, BLOCK>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
  }
}

template <bool NT, int UN, int BLOCK>
void launch_step_dtype(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  const StreamCount n = step_streams(grad_dtype, la, false);
  const Geometry gm = geometry_of(h, BLOCK * 4 * UN, BLOCK, n.wide, n.narrow);
  if (grad_dtype == NOVAK_GRAD_BF16) launch_step_la<unsigned short, u16x4, NT, UN, BLOCK>(la, gm, s, tb, c);
  else launch_step_la<float, f32x4, NT, UN, BLOCK>(la, gm, s, tb, c);
}

template <bool NT, int BLOCK>
void launch_step_un(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  switch (h->vec_per_lane) {
    case 1: launch_step_dtype<NT, 1, BLOCK>(h, grad_dtype, la, s, tb, c); break;
    case 2: launch_step_dtype<NT, 2, BLOCK>(h, grad_dtype, la, s, tb, c); break;
    default: launch_step_dtype<NT, 4, BLOCK>(h, grad_dtype, la, s, tb, c); break;
  }
}

template <bool NT>
void launch_step_block(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  switch (h->threads) {
    case 64: launch_step_un<NT, 64>(h, grad_dtype, la, s, tb, c); break;
    case 128: launch_step_un<NT, 128>(h, grad_dtype, la, s, tb, c); break;
    default: launch_step_un<NT, 256>(h, grad_dtype, la, s, tb, c); break;
  }
}

// Centralization, the bfloat16 first moment and the adaptive-beta moment updates are compiled into the default
// launch shape only (one wave64 per 256 elements).
template <typename GradS, typename GradV, bool NT, bool GC, typename MomS, typename MomV, bool AB>
void launch_step_special(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  const StreamCount n = step_streams(grad_dtype, la, sizeof(MomS) == 2);
  const Geometry gm = geometry_of(h, 256, 64, n.wide, n.narrow);
  const dim3 grid(gm.grid), block(64);
  switch (la) {
    case LA_OFF: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_OFF, NT, 1, 64, GC, MomS, MomV, AB>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_FIRST: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_FIRST, NT, 1, 64, GC, MomS, MomV, AB>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_MID: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_MID, NT, 1, 64, GC, MomS, MomV, AB>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    case LA_LAST_FUSED: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_LAST_FUSED, NT, 1, 64, GC, MomS, MomV, AB>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
    default: hipLaunchKernelGGL((novak_step_kernel<GradS, GradV, LA_BASIC_FUSED, NT, 1, 64, GC, MomS, MomV, AB>), grid, block, gm.lds, s, tb, c, gm.sub_shift); break;
  }
}

template <bool GC, typename MomS, typename MomV, bool AB>
void launch_step_special_dtype(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  if (grad_dtype == NOVAK_GRAD_BF16) {
    if (h->nontemporal) launch_step_special<unsigned short, u16x4, true, GC, MomS, MomV, AB>(h, grad_dtype, la, s, tb, c);
    else launch_step_special<unsigned short, u16x4, false, GC, MomS, MomV, AB>(h, grad_dtype, la, s, tb, c);
  } else {
    if (h->nontemporal) launch_step_special<float, f32x4, true, GC, MomS, MomV, AB>(h, grad_dtype, la, s, tb, c);
    else launch_step_special<float, f32x4, false, GC, MomS, MomV, AB>(h, grad_dtype, la, s, tb, c);
  }
}

template <bool GC, typename MomS, typename MomV>
void launch_step_special_ab(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  if (h->hp.adaptive_beta) launch_step_special_dtype<GC, MomS, MomV, true>(h, grad_dtype, la, s, tb, c);
  else launch_step_special_dtype<GC, MomS, MomV, false>(h, grad_dtype, la, s, tb, c);
}

void launch_step(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c) {
  const bool gc = (c.flags & F_GC) != 0;
  const bool bf16_m = h->hp.moment_dtype == NOVAK_MOMENT_BF16_M;
  if (gc && bf16_m) return launch_step_special_ab<true, unsigned short, u16x4>(h, grad_dtype, la, s, tb, c);
  if (bf16_m) return launch_step_special_ab<false, unsigned short, u16x4>(h, grad_dtype, la, s, tb, c);
  if (gc) return launch_step_special_ab<true, float, f32x4>(h, grad_dtype, la, s, tb, c);
  if (h->hp.adaptive_beta) return launch_step_special_dtype<false, float, f32x4, true>(h, grad_dtype, la, s, tb, c);
  if (h->nontemporal) launch_step_block<true>(h, grad_dtype, la, s, tb, c);
  else launch_step_block<false>(h, grad_dtype, la, s, tb, c);
}

// Device-step mode: the kernel that takes constants and lookahead phase from device memory (default shape).
template <typename GradS, typename GradV, int LA, bool NT, bool GC, bool AB>
void launch_step_device_ab(const LaunchCtx *h, const dim3 &grid, unsigned lds, int sub_shift, hipStream_t s, const Tables &tb) {
  if (h->hp.moment_dtype == NOVAK_MOMENT_BF16_M)
    hipLaunchKernelGGL((novak_step_device_kernel<GradS, GradV, LA, NT, GC, unsigned short, u16x4, AB>), grid, dim3(64), lds, s, tb, h->d_step, sub_shift);
  else
    hipLaunchKernelGGL((novak_step_device_kernel<GradS, GradV, LA, NT, GC, float, f32x4, AB>), grid, dim3(64), lds, s, tb, h->d_step, sub_shift);
}

template <typename GradS, typename GradV, int LA, bool NT, bool GC>
void launch_step_device_mom(const LaunchCtx *h, const dim3 &grid, unsigned lds, int sub_shift, hipStream_t s, const Tables &tb) {
  if (h->hp.adaptive_beta) launch_step_device_ab<GradS, GradV, LA, NT, GC, true>(h, grid, lds, sub_shift, s, tb);
  else launch_step_device_ab<GradS, GradV, LA, NT, GC, false>(h, grid, lds, sub_shift, s, tb);
}

template <typename GradS, typename GradV, int LA>
void launch_step_device_la(const LaunchCtx *h, const dim3 &grid, unsigned lds, int sub_shift, hipStream_t s, const Tables &tb) {
  const bool nt = h->nontemporal != 0, gc = h->n_gc > 0;
  if (nt && gc) launch_step_device_mom<GradS, GradV, LA, true, true>(h, grid, lds, sub_shift, s, tb);
  else if (nt) launch_step_device_mom<GradS, GradV, LA, true, false>(h, grid, lds, sub_shift, s, tb);
  else if (gc) launch_step_device_mom<GradS, GradV, LA, false, true>(h, grid, lds, sub_shift, s, tb);
  else launch_step_device_mom<GradS, GradV, LA, false, false>(h, grid, lds, sub_shift, s, tb);
}

template <typename GradS, typename GradV>
void launch_step_device_dtype(const LaunchCtx *h, const dim3 &grid, unsigned lds, int sub_shift, hipStream_t s, const Tables &tb) {
  switch (h->hp.lookahead_mode) {
    case NOVAK_LOOKAHEAD_MEMORY_EFFICIENT: launch_step_device_la<GradS, GradV, LA_RUNTIME_ME>(h, grid, lds, sub_shift, s, tb); break;
    case NOVAK_LOOKAHEAD_BASIC: launch_step_device_la<GradS, GradV, LA_RUNTIME_BASIC>(h, grid, lds, sub_shift, s, tb); break;
    default: launch_step_device_la<GradS, GradV, LA_OFF>(h, grid, lds, sub_shift, s, tb); break;
  }
}

void launch_step_device(const LaunchCtx *h, int grad_dtype, hipStream_t s, const Tables &tb) {
  // the host does not know the step's lookahead phase: residency for the phase with the most streams
  const int la = h->hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT ? LA_MID : LA_OFF;
  const StreamCount n = step_streams(grad_dtype, la, h->hp.moment_dtype == NOVAK_MOMENT_BF16_M);
  LaunchCtx shape = *h;                       // this kernel exists in the default launch shape only
  shape.vec_per_lane = 1;
  // With the run-time phase the kernel peaks two waves later than its host-step counterparts (11 instead of 9 per
  // compute unit with fp32 gradients, 12 with bfloat16 gradients: measured on the four multi-tensor lists).
  const double budget = h->hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT ? kDeviceStepBudget : kStepBudget;
  const Geometry gm = geometry_of(&shape, 256, 64, n.wide, n.narrow, budget);
  if (grad_dtype == NOVAK_GRAD_BF16) launch_step_device_dtype<unsigned short, u16x4>(h, dim3(gm.grid), gm.lds, gm.sub_shift, s, tb);
  else launch_step_device_dtype<float, f32x4>(h, dim3(gm.grid), gm.lds, gm.sub_shift, s, tb);
}

template <int OP, int BLOCK>
void launch_la_block(const LaunchCtx *h, hipStream_t s, const Tables &tb, float c0, float c1) {
  const Geometry gm = geometry_of(h, BLOCK * 4, BLOCK, OP == SYNC_BASIC ? 4 : 2);
  if (h->nontemporal) hipLaunchKernelGGL((novak_lookahead_kernel<OP, true, BLOCK>), dim3(gm.grid), dim3(BLOCK), gm.lds, s, tb, c0, c1, gm.sub_shift);
  else hipLaunchKernelGGL((novak_lookahead_kernel<OP, false, BLOCK>), dim3(gm.grid), dim3(BLOCK), gm.lds, s, tb, c0, c1, gm.sub_shift);
}

template <int OP>
void launch_la(const LaunchCtx *h, hipStream_t s, const Tables &tb, float c0, float c1) {
  switch (h->threads) {
    case 64: launch_la_block<OP, 64>(h, s, tb, c0, c1); break;
    case 128: launch_la_block<OP, 128>(h, s, tb, c0, c1); break;
    default: launch_la_block<OP, 256>(h, s, tb, c0, c1); break;
  }
}

template <bool NT, typename MomS, typename MomV>
void launch_apply(int la, const Geometry &gm, hipStream_t s, const Tables &tb, const Consts &c, const float *scale) {
  const dim3 grid(gm.grid), block(kScaledBlock);
  switch (la) {
    case LA_OFF: hipLaunchKernelGGL((novak_apply_kernel<LA_OFF, NT, MomS, MomV>), grid, block, gm.lds, s, tb, c, gm.sub_shift, scale); break;
    case LA_FIRST: hipLaunchKernelGGL((novak_apply_kernel<LA_FIRST, NT, MomS, MomV>), grid, block, gm.lds, s, tb, c, gm.sub_shift, scale); break;
    case LA_MID: hipLaunchKernelGGL((novak_apply_kernel<LA_MID, NT, MomS, MomV>), grid, block, gm.lds, s, tb, c, gm.sub_shift, scale); break;
    case LA_LAST_FUSED: hipLaunchKernelGGL((novak_apply_kernel<LA_LAST_FUSED, NT, MomS, MomV>), grid, block, gm.lds, s, tb, c, gm.sub_shift, scale); break;
    default: hipLaunchKernelGGL((novak_apply_kernel<LA_BASIC_FUSED, NT, MomS, MomV>), grid, block, gm.lds, s, tb, c, gm.sub_shift, scale); break;
  }
}

template <typename MomS, typename MomV, bool AB>
void launch_moments_ab(const LaunchCtx *h, int grad_dtype, const Geometry &g1, hipStream_t s, const Tables &tb, const Consts &c) {
  const dim3 grid1(g1.grid), block(kScaledBlock);
  const bool nt = h->nontemporal != 0;
  if (grad_dtype == NOVAK_GRAD_BF16) {
    if (nt) hipLaunchKernelGGL((novak_moments_kernel<unsigned short, u16x4, true, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, c, g1.sub_shift, h->d_partials);
    else hipLaunchKernelGGL((novak_moments_kernel<unsigned short, u16x4, false, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, c, g1.sub_shift, h->d_partials);
  } else {
    if (nt) hipLaunchKernelGGL((novak_moments_kernel<float, f32x4, true, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, c, g1.sub_shift, h->d_partials);
    else hipLaunchKernelGGL((novak_moments_kernel<float, f32x4, false, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, c, g1.sub_shift, h->d_partials);
  }
}

template <typename MomS, typename MomV>
void launch_moments(const LaunchCtx *h, int grad_dtype, const Geometry &g1, hipStream_t s, const Tables &tb, const Consts &c) {
  if (h->hp.adaptive_beta) launch_moments_ab<MomS, MomV, true>(h, grad_dtype, g1, s, tb, c);
  else launch_moments_ab<MomS, MomV, false>(h, grad_dtype, g1, s, tb, c);
}

// Gradient pre-pass: one read of the gradients gives each chunk's sum of squares (clipping) and the row sums
// (centralization); then the norm goes chunk sums -> tensor sums -> global factor in d_gscale, and the
// rows that span several waves get their means from the waves' partial sums.
// Residency: a read-only stream peaks at 6 resident waves of 16 KB per compute unit (10 - 12 waves of
// 8 KB with bf16 gradients); the LDS that bounds it doubles as the centralization's staging buffer.
template <typename GradS, typename GradV, bool NT>
void launch_prepass_kernel(bool norm, bool gc, const dim3 &grid, unsigned lds, hipStream_t s, const Tables &tb, int sub_shift,
                           NormSums *chunk_sums, RowPartial *row_partials) {
  const dim3 block(kScaledBlock);
  if (norm && gc) hipLaunchKernelGGL((novak_prepass_kernel<GradS, GradV, NT, true, true>), grid, block, lds, s, tb, sub_shift, chunk_sums, row_partials);
  else if (norm) hipLaunchKernelGGL((novak_prepass_kernel<GradS, GradV, NT, true, false>), grid, block, lds, s, tb, sub_shift, chunk_sums, row_partials);
  else hipLaunchKernelGGL((novak_prepass_kernel<GradS, GradV, NT, false, true>), grid, block, lds, s, tb, sub_shift, chunk_sums, row_partials);
}

hipError_t launch_prepass(const LaunchCtx *h, int grad_dtype, hipStream_t s, const Tables &tb) {
  const bool norm = clipping(h) || auto_only(h), gc = h->n_gc > 0;
  const bool bf16_g = grad_dtype == NOVAK_GRAD_BF16;
  Geometry g0;
  g0.sub_shift = log2_exact(h->chunk_elems / kPreSub);
  g0.grid = static_cast<unsigned>(h->n_chunks);          // one wave per chunk-table entry
  int waves = h->prepass_waves_per_cu ? h->prepass_waves_per_cu : (bf16_g ? (gc ? 10 : 12) : 6);
  unsigned lds = waves >= 32 ? 0u : (static_cast<unsigned>(h->lds_per_cu) / static_cast<unsigned>(waves)) & ~511u;
  if (lds > 65536u) lds = 65536u;
  if (gc && lds < kPreStageBytes) lds = kPreStageBytes;
  const dim3 grid(g0.grid);
  const bool nt = h->nontemporal != 0;
  if (bf16_g) {
    if (nt) launch_prepass_kernel<unsigned short, u16x4, true>(norm, gc, grid, lds, s, tb, g0.sub_shift, h->d_chunk_sums, h->d_row_partials);
    else launch_prepass_kernel<unsigned short, u16x4, false>(norm, gc, grid, lds, s, tb, g0.sub_shift, h->d_chunk_sums, h->d_row_partials);
  } else {
    if (nt) launch_prepass_kernel<float, f32x4, true>(norm, gc, grid, lds, s, tb, g0.sub_shift, h->d_chunk_sums, h->d_row_partials);
    else launch_prepass_kernel<float, f32x4, false>(norm, gc, grid, lds, s, tb, g0.sub_shift, h->d_chunk_sums, h->d_row_partials);
  }
  if (gc)
    hipLaunchKernelGGL(novak_rowfinal_kernel, dim3(static_cast<unsigned>((h->total_rows + 63) / 64)), dim3(64), 0, s, h->d_gc_tensor, h->d_row_first,
                       h->n_gc, h->d_gc, h->d_first_chunk, g0.sub_shift, h->total_rows, h->d_row_partials, h->d_row_means);
  if (norm) {
    ScaleParams sp;
    std::memset(&sp, 0, sizeof(sp));
    const int nt_count = h->n_tensors;
    hipLaunchKernelGGL(novak_reduce_tensors_kernel, dim3(static_cast<unsigned>(nt_count)), dim3(kTensorReduceBlock), 0, s, h->d_first_chunk, h->d_chunk_sums,
                       h->d_tensor_sums, h->d_scale, sp);
    if (clipping(h))
      hipLaunchKernelGGL(novak_clip_kernel, dim3(1), dim3(64), 0, s, nt_count, h->d_tensor_sums, static_cast<float>(h->hp.clip_threshold), h->d_gscale);
    if (auto_only(h)) {
      // the same kernel over the parameters (always fp32), then Eq. 20-22 from the two global norms
      Tables over_theta = tb;
      over_theta.grad = h->d_theta_ptrs;
      const int w_th = h->prepass_waves_per_cu ? h->prepass_waves_per_cu : 6;
      unsigned lds_th = w_th >= 32 ? 0u : (static_cast<unsigned>(h->lds_per_cu) / static_cast<unsigned>(w_th)) & ~511u;
      if (lds_th > 65536u) lds_th = 65536u;
      if (nt) launch_prepass_kernel<float, f32x4, true>(true, false, grid, lds_th, s, over_theta, g0.sub_shift, h->d_chunk_sums_theta, nullptr);
      else launch_prepass_kernel<float, f32x4, false>(true, false, grid, lds_th, s, over_theta, g0.sub_shift, h->d_chunk_sums_theta, nullptr);
      hipLaunchKernelGGL(novak_reduce_tensors_kernel, dim3(static_cast<unsigned>(nt_count)), dim3(kTensorReduceBlock), 0, s, h->d_first_chunk,
                         h->d_chunk_sums_theta, h->d_tensor_sums_theta, h->d_scale, sp);
      ScaleParams ap = sp;
      ap.auto_lo = static_cast<float>(h->hp.auto_clip_lo);
      ap.auto_hi = static_cast<float>(h->hp.auto_clip_hi);
      ap.gamma = h->hp.auto_lr_gamma;
      ap.auto_lr = 1;
      hipLaunchKernelGGL(novak_auto_lr_kernel, dim3(1), dim3(64), 0, s, nt_count, h->d_tensor_sums, h->d_scale, h->d_ema, ap,
                         h->d_tensor_sums_theta, h->d_ascale);
    }
  }
  return hipGetLastError();
}

// The two-pass step: moments + norm partials, fixed-order reductions, scaled apply.  `device_step`: constants and
// lookahead phase are in h->d_step (`la` is then the phase with the most streams, for the residency, and `c` unused).
template <typename MomS, typename MomV> void launch_moments_device(const LaunchCtx *, int, const Geometry &, hipStream_t, const Tables &);
template <typename MomS, typename MomV> void launch_apply_device_la(const LaunchCtx *, const Geometry &, hipStream_t, const Tables &);
hipError_t launch_scaled_step(const LaunchCtx *h, int grad_dtype, int la, hipStream_t s, const Tables &tb, const Consts &c, bool device_step = false) {
  const novak_hparams &hp = h->hp;
  const bool bf16_m = hp.moment_dtype == NOVAK_MOMENT_BF16_M;
  const bool bf16_g = grad_dtype == NOVAK_GRAD_BF16;
  // pass 1: theta, g, m, v read; m, v written
  const Geometry g1 = geometry_of(h, kScaledSub, kScaledBlock, 3 + (bf16_g ? 0 : 1) + (bf16_m ? 0 : 2), (bf16_g ? 1 : 0) + (bf16_m ? 2 : 0), kTwoPassBudget);
  const bool nt = h->nontemporal != 0;
  if (device_step) {
    if (bf16_m) launch_moments_device<unsigned short, u16x4>(h, grad_dtype, g1, s, tb);
    else launch_moments_device<float, f32x4>(h, grad_dtype, g1, s, tb);
  } else {
    if (bf16_m) launch_moments<unsigned short, u16x4>(h, grad_dtype, g1, s, tb, c);
    else launch_moments<float, f32x4>(h, grad_dtype, g1, s, tb, c);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ScaleParams sp;
  sp.trust_lo = static_cast<float>(hp.trust_clip_lo);
  sp.trust_hi = static_cast<float>(hp.trust_clip_hi);
  sp.auto_lo = static_cast<float>(hp.auto_clip_lo);
  sp.auto_hi = static_cast<float>(hp.auto_clip_hi);
  sp.gamma = hp.auto_lr_gamma;
  sp.layer_adaptation = hp.layer_adaptation;
  sp.auto_lr = hp.auto_lr;
  const int nt_count = h->n_tensors;
  hipLaunchKernelGGL(novak_reduce_chunks_kernel, dim3(static_cast<unsigned>(h->n_chunks)), dim3(64), 0, s, h->d_chunks, g1.sub_shift,
                     kScaledSub, h->d_partials, h->d_chunk_sums);
  hipLaunchKernelGGL(novak_reduce_tensors_kernel, dim3(static_cast<unsigned>(nt_count)), dim3(kTensorReduceBlock), 0, s, h->d_first_chunk, h->d_chunk_sums,
                     h->d_tensor_sums, h->d_scale, sp);
  if (hp.auto_lr)
    hipLaunchKernelGGL(novak_auto_lr_kernel, dim3(1), dim3(64), 0, s, nt_count, h->d_tensor_sums, h->d_scale, h->d_ema, sp,
                       static_cast<const NormSums *>(nullptr), static_cast<float *>(nullptr));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  int s2 = 3 + (bf16_m ? 0 : 1);                    // pass 2: theta, m, v read; theta written
  if (la_reads(la)) s2 += 1;
  if (la_writes(la)) s2 += 1;
  const Geometry g2 = geometry_of(h, kScaledSub, kScaledBlock, s2, bf16_m ? 1 : 0, kTwoPassBudget);
  if (device_step) {
    if (bf16_m) launch_apply_device_la<unsigned short, u16x4>(h, g2, s, tb);
    else launch_apply_device_la<float, f32x4>(h, g2, s, tb);
  } else if (bf16_m) {
    if (nt) launch_apply<true, unsigned short, u16x4>(la, g2, s, tb, c, h->d_scale);
    else launch_apply<false, unsigned short, u16x4>(la, g2, s, tb, c, h->d_scale);
  } else {
    if (nt) launch_apply<true, float, f32x4>(la, g2, s, tb, c, h->d_scale);
    else launch_apply<false, float, f32x4>(la, g2, s, tb, c, h->d_scale);
  }
  return hipGetLastError();
}

// The two-pass step in device-step mode: constants and lookahead phase come from the record the prologue kernel wrote.
template <int LA, typename MomS, typename MomV>
void launch_apply_device(const LaunchCtx *h, const Geometry &gm, hipStream_t s, const Tables &tb) {
  const dim3 grid(gm.grid), block(kScaledBlock);
  if (h->nontemporal) hipLaunchKernelGGL((novak_apply_device_kernel<LA, true, MomS, MomV>), grid, block, gm.lds, s, tb, h->d_step, gm.sub_shift, h->d_scale);
  else hipLaunchKernelGGL((novak_apply_device_kernel<LA, false, MomS, MomV>), grid, block, gm.lds, s, tb, h->d_step, gm.sub_shift, h->d_scale);
}

template <typename MomS, typename MomV>
void launch_apply_device_la(const LaunchCtx *h, const Geometry &gm, hipStream_t s, const Tables &tb) {
  switch (h->hp.lookahead_mode) {
    case NOVAK_LOOKAHEAD_MEMORY_EFFICIENT: launch_apply_device<LA_RUNTIME_ME, MomS, MomV>(h, gm, s, tb); break;
    case NOVAK_LOOKAHEAD_BASIC: launch_apply_device<LA_RUNTIME_BASIC, MomS, MomV>(h, gm, s, tb); break;
    default: launch_apply_device<LA_OFF, MomS, MomV>(h, gm, s, tb); break;
  }
}

template <typename MomS, typename MomV, bool AB>
void launch_moments_device_ab(const LaunchCtx *h, int grad_dtype, const Geometry &g1, hipStream_t s, const Tables &tb) {
  const dim3 grid1(g1.grid), block(kScaledBlock);
  const bool nt = h->nontemporal != 0;
  if (grad_dtype == NOVAK_GRAD_BF16) {
    if (nt) hipLaunchKernelGGL((novak_moments_device_kernel<unsigned short, u16x4, true, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, h->d_step, g1.sub_shift, h->d_partials);
    else hipLaunchKernelGGL((novak_moments_device_kernel<unsigned short, u16x4, false, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, h->d_step, g1.sub_shift, h->d_partials);
  } else {
    if (nt) hipLaunchKernelGGL((novak_moments_device_kernel<float, f32x4, true, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, h->d_step, g1.sub_shift, h->d_partials);
    else hipLaunchKernelGGL((novak_moments_device_kernel<float, f32x4, false, MomS, MomV, AB>), grid1, block, g1.lds, s, tb, h->d_step, g1.sub_shift, h->d_partials);
  }
}

template <typename MomS, typename MomV>
void launch_moments_device(const LaunchCtx *h, int grad_dtype, const Geometry &g1, hipStream_t s, const Tables &tb) {
  if (h->hp.adaptive_beta) launch_moments_device_ab<MomS, MomV, true>(h, grad_dtype, g1, s, tb);
  else launch_moments_device_ab<MomS, MomV, false>(h, grad_dtype, g1, s, tb);
}

hipError_t launch_sync(const LaunchCtx *h, hipStream_t s) {
  if (h->n_chunks == 0) return hipSuccess;
  const Tables tb = tables_of(h);
  if (h->hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT) {
    launch_la<SYNC_ME>(h, s, tb, 0.0f, 0.0f);
  } else {
    const float c1 = static_cast<float>(h->hp.la_alpha);
    const float c0 = static_cast<float>(1.0 - h->hp.la_alpha);
    launch_la<SYNC_BASIC>(h, s, tb, c0, c1);
  }
  return hipGetLastError();
}

// Enqueues every kernel of one step on `stream`: the gradient pre-passes, the single-pass or two-pass
// update, and the separate sync where the plan asks for one.  The tables of `cx` (gradient pointers
// included) must already be in place in stream order.
hipError_t enqueue_step(const LaunchCtx *cx, int grad_dtype, const StepPlan &pl, hipStream_t stream) {
  if (cx->n_chunks == 0) return hipSuccess;
  Consts c = pl.c;
  hipError_t e;
  if (cx->n_gc > 0) c.flags |= F_GC;
  if (auto_only(cx)) c.flags |= F_AUTO;
  if ((clipping(cx) || cx->n_gc > 0 || auto_only(cx)) && (e = launch_prepass(cx, grad_dtype, stream, tables_of(cx))) != hipSuccess) return e;
  if (two_pass(cx)) {
    if ((e = launch_scaled_step(cx, grad_dtype, pl.la, stream, tables_of(cx), c)) != hipSuccess) return e;
  } else {
    launch_step(cx, grad_dtype, pl.la, stream, tables_of(cx), c);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (pl.sync_after) return launch_sync(cx, stream);
  return hipSuccess;
}

// The same in device-step mode: a prologue kernel (when asked for) reads the caller's counter and writes the constants
// and lookahead phase, then the kernels follow; which of them run does not depend on t.
hipError_t enqueue_step_device(const LaunchCtx *cx, int grad_dtype, hipStream_t stream, int n_records) {
  hipError_t e;
  const uint32_t extra = (cx->n_gc > 0 ? F_GC : 0u) | (auto_only(cx) ? F_AUTO : 0u);
  if (n_records > 0) {      // cx->d_step is the first of the n_records slots to fill
    hipLaunchKernelGGL(novak_prologue_kernel, dim3(1), dim3(kDeviceRing), 0, stream, cx->hp, extra, cx->d_counter, cx->d_step, n_records);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (cx->n_chunks == 0) {                           // a list without elements: the step still counts
    hipLaunchKernelGGL(novak_count_kernel, dim3(1), dim3(64), 0, stream, cx->d_step);
    return hipGetLastError();
  }
  if ((clipping(cx) || cx->n_gc > 0 || auto_only(cx)) && (e = launch_prepass(cx, grad_dtype, stream, tables_of(cx))) != hipSuccess) return e;
  if (two_pass(cx)) {
    // the host does not know the step's lookahead phase: residency for the phase with the most streams
    const int la = cx->hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT ? LA_MID : LA_OFF;
    if ((e = launch_scaled_step(cx, grad_dtype, la, stream, tables_of(cx), Consts(), true)) != hipSuccess) return e;
  } else {
    launch_step_device(cx, grad_dtype, stream, tables_of(cx));
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // a window of one step: the sync follows every step as its own kernel
  if (cx->hp.lookahead_mode == NOVAK_LOOKAHEAD_MEMORY_EFFICIENT && cx->hp.la_k == 1) return launch_sync(cx, stream);
  return hipSuccess;
}

// A launch is limited to 2^32 - 1 threads.  At the finest decomposition (one wave64 per 256 elements) a list
// whose chunks cover `covered` elements needs covered / 4 threads.
bool fits_one_launch(int64_t n_chunks, int64_t chunk_elems) {
  return n_chunks <= (int64_t{0xffffffffLL} / 64) / (chunk_elems / kMinSub);
}

// The chunk-table entry size a list starts with.  Without a gradient pre-pass: NOVAK_CHUNK_DEFAULT (the step kernels do
// not depend on it).  With one (one wave per entry, 6 resident per compute unit): the largest of 65536 / 16384 / 4096
// elements that still gives the pre-pass four rounds of waves.  Long entries amortise a wave's start-up (1.3e9
// parameters: +1.0 ... 1.6 % of the whole step at 65536 against 16384); a short list needs the waves more: with
// centralization its pre-pass waves are chains of latency-bound row reductions, and one round of them took 80 us where
// four rounds of a quarter the size take 27 (2.6e7 parameters: +32 % at 4096).  `max_chunks` bounds the table (the
// allocation-free step's static array); the handle path and that step share this function, so the same list is cut
// the same way by both.
int64_t initial_chunk_elems(const novak_tensor_desc *tensors, int32_t n_tensors, bool prepass, int32_t device_id, int64_t max_chunks) {
  if (!prepass) return NOVAK_CHUNK_DEFAULT;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device_id) != hipSuccess || cus < 1) {
    (void)hipGetLastError();
    cus = 256;
  }
  const int64_t rounds_of_four = int64_t{4} * 6 * cus;
  int64_t pick = NOVAK_CHUNK_DEFAULT;
  for (const int64_t c : {int64_t{65536}, int64_t{16384}, int64_t{4096}}) {
    int64_t planned = 0;
    for (int32_t i = 0; i < n_tensors; ++i) planned += (tensors[i].numel + c - 1) / c;
    if (planned > max_chunks || !fits_one_launch(planned, c)) continue;
    pick = c;
    if (planned >= rounds_of_four) break;
  }
  return pick;
}

// Descriptor checks shared by novak_create and the allocation-free step.  On failure writes the reason.
int check_descs(const novak_hparams &eff, const novak_tensor_desc *tensors, int32_t n_tensors, std::string *why) {
  for (int32_t i = 0; i < n_tensors; ++i) {
    const novak_tensor_desc &d = tensors[i];
    const std::string who = "tensor " + std::to_string(i);
    if (d.numel < 0) { *why = who + ": numel < 0"; return NOVAK_ERR_INVALID_ARG; }
    if (d.numel == 0) continue;
    if (!d.param || !d.exp_avg || !d.exp_avg_sq) { *why = who + ": param/exp_avg/exp_avg_sq is NULL"; return NOVAK_ERR_NULL_POINTER; }
    if (eff.lookahead_mode != NOVAK_LOOKAHEAD_NONE && !d.la_buf) { *why = who + ": la_buf is NULL with lookahead on"; return NOVAK_ERR_NULL_POINTER; }
    const uintptr_t bits = reinterpret_cast<uintptr_t>(d.param) | reinterpret_cast<uintptr_t>(d.exp_avg_sq) | reinterpret_cast<uintptr_t>(d.la_buf);
    if (bits & 3u) { *why = who + ": pointer not 4-byte aligned"; return NOVAK_ERR_MISALIGNED; }
    if (reinterpret_cast<uintptr_t>(d.exp_avg) & (eff.moment_dtype == NOVAK_MOMENT_BF16_M ? 1u : 3u)) {
      *why = who + ": exp_avg not aligned to its element size";
      return NOVAK_ERR_MISALIGNED;
    }
    if (eff.use_gc && (d.rows < 0 || (d.rows > 0 && d.numel % d.rows != 0))) {
      *why = who + ": rows must be >= 0 and divide numel";
      return NOVAK_ERR_INVALID_ARG;
    }
  }
  return NOVAK_OK;
}

int check_grads(const novak_tensor_desc *tensors, size_t n, void *const *grads, int32_t grad_dtype, std::string *why) {
  if (n > 0 && !grads) { *why = "grads is NULL"; return NOVAK_ERR_NULL_POINTER; }
  if (grad_dtype != NOVAK_GRAD_F32 && grad_dtype != NOVAK_GRAD_BF16) { *why = "unknown grad_dtype"; return NOVAK_ERR_INVALID_ARG; }
  const uintptr_t amask = grad_dtype == NOVAK_GRAD_BF16 ? 1u : 3u;
  for (size_t i = 0; i < n; ++i) {
    if (tensors[i].numel == 0) continue;
    if (!grads[i]) { *why = "grads[" + std::to_string(i) + "] is NULL"; return NOVAK_ERR_NULL_POINTER; }
    if (reinterpret_cast<uintptr_t>(grads[i]) & amask) { *why = "grads[" + std::to_string(i) + "] not aligned to its element size"; return NOVAK_ERR_MISALIGNED; }
  }
  return NOVAK_OK;
}

// No exception leaves the library: what can throw on the host side of an entry point is an allocation (an error
// string, a staging vector), which becomes a status code.
template <typename F>
int guarded(F &&body) {
  try {
    return body();
  } catch (...) {
    return NOVAK_ERR_NO_MEMORY;
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// entry points
// ------------------------------------------------------------------------------------------------
extern "C" {

static int create_impl(novak_handle **out, const novak_hparams *hp, const novak_tensor_desc *tensors, int32_t n_tensors,
                       int32_t device_id) {
  if (!out) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "out is NULL");
  *out = nullptr;
  if (!hp) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "hp is NULL");
  if (n_tensors < 0) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "n_tensors < 0");
  if (n_tensors > 0 && !tensors) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "tensors is NULL");
  if (device_id < 0) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "device_id < 0");
  novak_hparams eff;
  uint32_t warn = 0;
  int rc = novak_validate_hparams(hp, &eff, &warn);
  if (rc != NOVAK_OK) return fail(nullptr, rc, "hyper-parameters rejected (section 5.8 validation rules)");
  if (eff.device_step) {
    if (eff.lookahead_mode != NOVAK_LOOKAHEAD_NONE && !eff.auto_sync)
      return fail(nullptr, NOVAK_ERR_INVALID_ARG, "device_step with lookahead needs auto_sync = 1 (the host does not know when a sync is due)");
  }
  std::string why;
  rc = check_descs(eff, tensors, n_tensors, &why);
  if (rc != NOVAK_OK) return fail(nullptr, rc, why);
  {  // refuse, before anything touches the device, a list that one launch cannot cover
    int64_t planned = 0;
    std::vector<int64_t> sizes(static_cast<size_t>(n_tensors));
    for (int32_t i = 0; i < n_tensors; ++i) sizes[static_cast<size_t>(i)] = tensors[i].numel;
    rc = novak_plan_chunks(sizes.data(), n_tensors, NOVAK_CHUNK_DEFAULT, nullptr, 0, &planned);
    if (rc != NOVAK_OK) return fail(nullptr, rc, "chunk planning failed");
    if (!fits_one_launch(planned, NOVAK_CHUNK_DEFAULT)) return fail(nullptr, NOVAK_ERR_INVALID_ARG, kTooLarge);
  }

  novak_handle *h = new (std::nothrow) novak_handle();
  if (!h) return fail(nullptr, NOVAK_ERR_NO_MEMORY, "host allocation failed");
  struct Guard {                     // releases the half-built handle on every early exit, exceptions included
    novak_handle *h;
    ~Guard() { if (h) novak_destroy(h); }
  } guard{h};
  h->hp = eff;
  h->warnings = warn;
  h->device_id = device_id;
  h->n_tensors = n_tensors;
  h->tensors.assign(tensors, tensors + n_tensors);
  h->numels.resize(static_cast<size_t>(n_tensors));
  for (int32_t i = 0; i < n_tensors; ++i) {
    h->numels[static_cast<size_t>(i)] = tensors[i].numel;
    h->total_numel += tensors[i].numel;
  }
  h->last_grads.assign(static_cast<size_t>(n_tensors), nullptr);

  auto bail = [&](int status) {
    g_create_error = h->error;
    return status;
  };
  DeviceScope scope;
  hipError_t e = scope.enter(device_id);
  if (e != hipSuccess) return bail(fail_hip(h, e, "hipSetDevice"));
  int lds_cu = 0;
  if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device_id) == hipSuccess && lds_cu >= 65536)
    h->lds_per_cu = lds_cu;
  if (eff.device_step && (e = hipMalloc(reinterpret_cast<void **>(&h->d_ring), kDeviceRing * sizeof(DeviceStep))) != hipSuccess)
    return bail(fail_hip(h, e, "hipMalloc(device step records)"));
  if (n_tensors > 0) {
    const size_t n = static_cast<size_t>(n_tensors);
    const size_t bytes = 5 * n * sizeof(void *);
    if ((e = hipMalloc(&h->d_ptrs, bytes)) != hipSuccess) return bail(fail_hip(h, e, "hipMalloc(pointer tables)"));
    std::vector<void *> host(5 * n, nullptr);
    for (size_t i = 0; i < n; ++i) {
      host[4 * i + 0] = tensors[i].param;      // TensorPtrs record i
      host[4 * i + 1] = tensors[i].exp_avg;
      host[4 * i + 2] = tensors[i].exp_avg_sq;
      host[4 * i + 3] = tensors[i].la_buf;
    }
    if ((e = hipMemcpy(h->d_ptrs, host.data(), bytes, hipMemcpyHostToDevice)) != hipSuccess) return bail(fail_hip(h, e, "hipMemcpy(pointer tables)"));
    if ((e = hipMalloc(reinterpret_cast<void **>(&h->d_out_ptrs), n * sizeof(float *))) != hipSuccess) return bail(fail_hip(h, e, "hipMalloc(output pointers)"));
    if (auto_only(h)) {      // the parameters' pointers as a plain list, for the pre-pass that takes their norm
      std::vector<const void *> th(n, nullptr);
      for (size_t i = 0; i < n; ++i) th[i] = tensors[i].param;
      if ((e = hipMalloc(reinterpret_cast<void **>(&h->d_theta_ptrs), n * sizeof(void *))) != hipSuccess) return bail(fail_hip(h, e, "hipMalloc(parameter pointers)"));
      if ((e = hipMemcpy(h->d_theta_ptrs, th.data(), n * sizeof(void *), hipMemcpyHostToDevice)) != hipSuccess) return bail(fail_hip(h, e, "hipMemcpy(parameter pointers)"));
    }
    if ((e = hipHostMalloc(reinterpret_cast<void **>(&h->h_ring), (novak_handle::kRing + 1) * n * sizeof(void *), hipHostMallocDefault)) != hipSuccess)
      return bail(fail_hip(h, e, "hipHostMalloc(pointer staging ring)"));
    for (int r = 0; r < novak_handle::kRing; ++r)
      if ((e = hipEventCreateWithFlags(&h->ring_ev[r], hipEventDisableTiming)) != hipSuccess) return bail(fail_hip(h, e, "hipEventCreate"));
    if ((e = hipEventCreateWithFlags(&h->out_ev, hipEventDisableTiming)) != hipSuccess) return bail(fail_hip(h, e, "hipEventCreate"));
  }
  if (eff.use_gc && n_tensors > 0) {
    const size_t n = static_cast<size_t>(n_tensors);
    std::vector<GcInfo> info(n);
    std::vector<int> list;
    std::vector<int64_t> first(1, 0);
    for (size_t i = 0; i < n; ++i) {
      info[i].cols = 0; info[i].inv_cols = 0.0; info[i].means = nullptr;
      if (tensors[i].rows >= 1 && tensors[i].numel > 0) {
        list.push_back(static_cast<int>(i));
        first.push_back(first.back() + tensors[i].rows);
      }
    }
    h->n_gc = static_cast<int>(list.size());
    h->total_rows = first.back();
    if (h->total_rows > 0x7fffffffLL) return bail(fail(h, NOVAK_ERR_INVALID_ARG, "too many rows to centralize in one launch"));
    if (h->n_gc > 0) {
      if ((e = hipMalloc(reinterpret_cast<void **>(&h->d_row_means), static_cast<size_t>(h->total_rows) * sizeof(double))) != hipSuccess)
        return bail(fail_hip(h, e, "hipMalloc(row means)"));
      for (size_t j = 0; j < list.size(); ++j) {
        const size_t i = static_cast<size_t>(list[j]);
        info[i].cols = tensors[i].numel / tensors[i].rows;
        info[i].inv_cols = 1.0 / static_cast<double>(info[i].cols);
        info[i].means = h->d_row_means + first[j];
      }
      if ((e = hipMalloc(reinterpret_cast<void **>(&h->d_gc), n * sizeof(GcInfo))) != hipSuccess ||
          (e = hipMemcpy(h->d_gc, info.data(), n * sizeof(GcInfo), hipMemcpyHostToDevice)) != hipSuccess ||
          (e = hipMalloc(reinterpret_cast<void **>(&h->d_gc_tensor), list.size() * sizeof(int))) != hipSuccess ||
          (e = hipMemcpy(h->d_gc_tensor, list.data(), list.size() * sizeof(int), hipMemcpyHostToDevice)) != hipSuccess ||
          (e = hipMalloc(reinterpret_cast<void **>(&h->d_row_first), first.size() * sizeof(int64_t))) != hipSuccess ||
          (e = hipMemcpy(h->d_row_first, first.data(), first.size() * sizeof(int64_t), hipMemcpyHostToDevice)) != hipSuccess)
        return bail(fail_hip(h, e, "gradient-centralization tables"));
    }
  }
  h->chunk_elems = initial_chunk_elems(tensors, n_tensors, clipping(h) || h->n_gc > 0 || auto_only(h), device_id, INT64_MAX);
  rc = build_chunk_table(h);
  if (rc != NOVAK_OK) return bail(rc);
  guard.h = nullptr;
  *out = h;
  return NOVAK_OK;
}

// No exception leaves the library: host allocation failures become status codes.
int novak_create(novak_handle **out, const novak_hparams *hp, const novak_tensor_desc *tensors, int32_t n_tensors,
                 int32_t device_id) {
  try {
    return create_impl(out, hp, tensors, n_tensors, device_id);
  } catch (const std::bad_alloc &) {
    if (out) *out = nullptr;
    g_create_error.clear();
    return NOVAK_ERR_NO_MEMORY;
  } catch (...) {
    if (out) *out = nullptr;
    g_create_error.clear();
    return NOVAK_ERR_INVALID_ARG;
  }
}

static int arena_alloc_impl(int32_t device_id, size_t bytes, void **ptr, int32_t *contiguous) {
  if (!ptr) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "ptr is NULL");
  *ptr = nullptr;
  if (contiguous) *contiguous = 0;
  if (device_id < 0 || bytes == 0) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "device_id < 0 or bytes == 0");
  DeviceScope scope;
  hipError_t e = scope.enter(device_id);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipSetDevice");
  void *p = nullptr;
  e = hipExtMallocWithFlags(&p, bytes, hipDeviceMallocContiguous);
  if (e == hipSuccess && p) {
    if (contiguous) *contiguous = 1;
  } else {
    (void)hipGetLastError();          // the refusal is not an error of this call: fall back
    p = nullptr;
    e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return fail_hip(nullptr, e, "hipMalloc(arena)");
  }
  *ptr = p;
  return NOVAK_OK;
}

static int arena_free_impl(int32_t device_id, void *ptr) {
  if (!ptr) return NOVAK_OK;
  if (device_id < 0) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "device_id < 0");
  DeviceScope scope;
  hipError_t e = scope.enter(device_id);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipSetDevice");
  e = hipFree(ptr);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipFree(arena)");
  return NOVAK_OK;
}

// ---- allocator hooks for torch.cuda.memory.CUDAPluggableAllocator / torch.cuda.MemPool ----------------------
namespace {
struct TorchBlock {
  void *base;
  bool contiguous;
};
std::mutex g_torch_mutex;
std::unordered_map<void *, TorchBlock> g_torch_blocks;     // returned address -> what to free
unsigned g_torch_large_count = 0;
constexpr ptrdiff_t kTorchLarge = ptrdiff_t{1} << 20;
}  // namespace

void *novak_torch_malloc(ptrdiff_t size, int device, void * /*stream*/) {
  if (size < 0 || device < 0) return nullptr;
  if (size == 0) size = 1;
  try {
    DeviceScope scope;
    if (scope.enter(device) != hipSuccess) return nullptr;
    TorchBlock blk{nullptr, false};
    size_t skew = 0;
    if (size >= kTorchLarge) {
      {
        std::lock_guard<std::mutex> lock(g_torch_mutex);
        skew = (static_cast<size_t>(g_torch_large_count++) * NOVAK_ARENA_ROLE_SKEW) % NOVAK_ARENA_ROLE_PERIOD;
      }
      const size_t bytes = static_cast<size_t>(size) + NOVAK_ARENA_ROLE_PERIOD;
      if (hipExtMallocWithFlags(&blk.base, bytes, hipDeviceMallocContiguous) == hipSuccess && blk.base) {
        blk.contiguous = true;
      } else {
        (void)hipGetLastError();
        blk.base = nullptr;
        if (hipMalloc(&blk.base, bytes) != hipSuccess) {
          (void)hipGetLastError();
          return nullptr;
        }
      }
    } else if (hipMalloc(&blk.base, static_cast<size_t>(size)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    void *ret = static_cast<char *>(blk.base) + skew;
    std::lock_guard<std::mutex> lock(g_torch_mutex);
    g_torch_blocks[ret] = blk;
    return ret;
  } catch (...) {
    return nullptr;
  }
}

void novak_torch_free(void *ptr, ptrdiff_t /*size*/, int device, void * /*stream*/) {
  if (!ptr) return;
  TorchBlock blk{ptr, false};
  {
    std::lock_guard<std::mutex> lock(g_torch_mutex);
    auto it = g_torch_blocks.find(ptr);
    if (it == g_torch_blocks.end()) return;        // not ours: leave it alone
    blk = it->second;
    g_torch_blocks.erase(it);
  }
  DeviceScope scope;
  if (device >= 0) (void)scope.enter(device);
  (void)hipFree(blk.base);
}

void novak_torch_alloc_stats(int64_t *live, int64_t *live_contiguous) {
  std::lock_guard<std::mutex> lock(g_torch_mutex);
  int64_t n = 0, c = 0;
  for (const auto &kv : g_torch_blocks) {
    ++n;
    if (kv.second.contiguous) ++c;
  }
  if (live) *live = n;
  if (live_contiguous) *live_contiguous = c;
}

int novak_destroy(novak_handle *h) {
  if (!h) return NOVAK_OK;
  DeviceScope scope;
  (void)scope.enter(h->device_id);
  free_device_tables(h);
  if (h->d_ptrs) (void)hipFree(h->d_ptrs);
  if (h->d_ring) (void)hipFree(h->d_ring);
  if (h->d_out_ptrs) (void)hipFree(h->d_out_ptrs);
  if (h->d_theta_ptrs) (void)hipFree(h->d_theta_ptrs);
  if (h->d_gc) (void)hipFree(h->d_gc);
  if (h->d_gc_tensor) (void)hipFree(h->d_gc_tensor);
  if (h->d_row_first) (void)hipFree(h->d_row_first);
  if (h->d_row_means) (void)hipFree(h->d_row_means);
  if (h->h_ring) (void)hipHostFree(h->h_ring);
  for (int r = 0; r < novak_handle::kRing; ++r)
    if (h->ring_ev[r]) (void)hipEventDestroy(h->ring_ev[r]);
  if (h->out_ev) (void)hipEventDestroy(h->out_ev);
  delete h;
  return NOVAK_OK;
}

int novak_get_info(const novak_handle *h, novak_info *info) {
  if (!h || !info) return NOVAK_ERR_NULL_POINTER;
  if (info->struct_size != sizeof(novak_info)) return NOVAK_ERR_INVALID_ARG;
  info->nesterov_mode = h->hp.nesterov_mode;
  info->lookahead_mode = h->hp.lookahead_mode;
  info->warnings = h->warnings;
  info->n_tensors = static_cast<int32_t>(h->tensors.size());
  info->n_chunks = h->n_chunks;
  info->chunk_elems = h->chunk_elems;
  info->total_numel = h->total_numel;
  info->last_step = h->last_step;
  info->sync_due = h->sync_due;
  info->device_id = h->device_id;
  info->layer_adaptation = h->hp.layer_adaptation;
  info->auto_lr = h->hp.auto_lr;
  info->use_gc = h->hp.use_gc;
  info->moment_dtype = h->hp.moment_dtype;
  info->n_centralized = h->n_gc;
  return NOVAK_OK;
}

static int nesterov_extrapolate_impl(novak_handle *h, void *const *out, void *hip_stream) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (h->broken) return fail(h, NOVAK_ERR_STATE, "the handle lost its tables in a failed novak_set_tuning; destroy it");
  const size_t n = h->tensors.size();
  if (n > 0 && !out) return fail(h, NOVAK_ERR_NULL_POINTER, "out is NULL");
  for (size_t i = 0; i < n; ++i) {
    if (h->numels[i] == 0) continue;
    if (!out[i]) return fail(h, NOVAK_ERR_NULL_POINTER, "out[" + std::to_string(i) + "] is NULL");
    if (reinterpret_cast<uintptr_t>(out[i]) & 3u) return fail(h, NOVAK_ERR_MISALIGNED, "out[" + std::to_string(i) + "] not 4-byte aligned");
  }
  if (h->n_chunks == 0) return NOVAK_OK;
  DeviceScope scope;
  NOVAK_HIP(h, scope.enter(h->device_id));
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // the list is staged in pinned memory owned by the handle, so the caller's array may be reused as
  // soon as this returns; the slot is rewritten only after the previous call's copy has executed
  if (h->out_used) NOVAK_HIP(h, hipEventSynchronize(h->out_ev));
  void **staged = h->h_ring + static_cast<size_t>(novak_handle::kRing) * n;
  std::memcpy(staged, out, n * sizeof(void *));
  NOVAK_HIP(h, hipMemcpyAsync(h->d_out_ptrs, staged, n * sizeof(float *), hipMemcpyHostToDevice, stream));
  NOVAK_HIP(h, hipEventRecord(h->out_ev, stream));
  h->out_used = true;
  const bool bf16_m_out = h->hp.moment_dtype == NOVAK_MOMENT_BF16_M;
  const Geometry gm = geometry_of(h, 256, 64, bf16_m_out ? 2 : 3, bf16_m_out ? 1 : 0);
  const float bn = static_cast<float>(h->hp.beta_n);
  const dim3 grid(gm.grid), block(64);
  if (h->hp.moment_dtype == NOVAK_MOMENT_BF16_M) {
    if (h->nontemporal) hipLaunchKernelGGL((novak_extrapolate_kernel<true, unsigned short, u16x4>), grid, block, gm.lds, stream, tables_of(h), h->d_out_ptrs, bn, gm.sub_shift);
    else hipLaunchKernelGGL((novak_extrapolate_kernel<false, unsigned short, u16x4>), grid, block, gm.lds, stream, tables_of(h), h->d_out_ptrs, bn, gm.sub_shift);
  } else {
    if (h->nontemporal) hipLaunchKernelGGL((novak_extrapolate_kernel<true, float, f32x4>), grid, block, gm.lds, stream, tables_of(h), h->d_out_ptrs, bn, gm.sub_shift);
    else hipLaunchKernelGGL((novak_extrapolate_kernel<false, float, f32x4>), grid, block, gm.lds, stream, tables_of(h), h->d_out_ptrs, bn, gm.sub_shift);
  }
  NOVAK_HIP(h, hipGetLastError());
  return NOVAK_OK;
}

static int set_auto_lr_state_impl(novak_handle *h, void *ema) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (!h->hp.auto_lr) return fail(h, NOVAK_ERR_STATE, "auto_lr is off (or was disabled by the fast path)");
  if (!ema) return fail(h, NOVAK_ERR_NULL_POINTER, "ema is NULL");
  if (reinterpret_cast<uintptr_t>(ema) & 7u) return fail(h, NOVAK_ERR_MISALIGNED, "ema must be 8-byte aligned");
  h->d_ema = static_cast<double *>(ema);
  return NOVAK_OK;
}

static int set_step_counter_impl(novak_handle *h, void *counter) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (!h->hp.device_step) return fail(h, NOVAK_ERR_STATE, "the handle counts steps on the host (device_step is off)");
  if (!counter) return fail(h, NOVAK_ERR_NULL_POINTER, "counter is NULL");
  if (reinterpret_cast<uintptr_t>(counter) & 7u) return fail(h, NOVAK_ERR_MISALIGNED, "counter must be 8-byte aligned");
  h->d_counter = static_cast<int64_t *>(counter);
  return NOVAK_OK;
}

static int copy_tensor_scales_impl(novak_handle *h, float *out, void *hip_stream) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (h->broken) return fail(h, NOVAK_ERR_STATE, "the handle lost its tables in a failed novak_set_tuning; destroy it");
  if (!scaled(h)) return fail(h, NOVAK_ERR_STATE, "neither layer adaptation nor auto-LR is on: there are no per-tensor scales");
  if (h->tensors.empty()) return NOVAK_OK;
  if (!out) return fail(h, NOVAK_ERR_NULL_POINTER, "out is NULL");
  DeviceScope scope;
  NOVAK_HIP(h, scope.enter(h->device_id));
  NOVAK_HIP(h, hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  NOVAK_HIP(h, hipMemcpy(out, h->d_scale, h->tensors.size() * sizeof(float), hipMemcpyDeviceToHost));
  return NOVAK_OK;
}

const char *novak_last_error(const novak_handle *h) { return h ? h->error.c_str() : g_create_error.c_str(); }

static int set_tuning_impl(novak_handle *h, int32_t key, int64_t value) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (key == NOVAK_TUNE_NONTEMPORAL) {
    h->nontemporal = value ? 1 : 0;
    return NOVAK_OK;
  }
  if (key == NOVAK_TUNE_WAVES_PER_CU) {
    if (value < 0 || value > 32) return fail(h, NOVAK_ERR_INVALID_ARG, "waves_per_cu must be in [0, 32]");
    h->waves_per_cu = static_cast<int>(value);
    return NOVAK_OK;
  }
  if (key == NOVAK_TUNE_PREPASS_WAVES_PER_CU) {
    if (value < 0 || value > 32) return fail(h, NOVAK_ERR_INVALID_ARG, "prepass_waves_per_cu must be in [0, 32]");
    h->prepass_waves_per_cu = static_cast<int>(value);
    return NOVAK_OK;
  }
  if (key == NOVAK_TUNE_THREADS) {
    if (value != 64 && value != 128 && value != 256) return fail(h, NOVAK_ERR_INVALID_ARG, "threads must be 64, 128 or 256");
    h->threads = static_cast<int>(value);
    return NOVAK_OK;
  }
  if (key == NOVAK_TUNE_VEC_PER_LANE) {
    if (value != 1 && value != 2 && value != 4) return fail(h, NOVAK_ERR_INVALID_ARG, "vec_per_lane must be 1, 2 or 4");
    h->vec_per_lane = static_cast<int>(value);
    return NOVAK_OK;
  }
  if (key == NOVAK_TUNE_CHUNK_ELEMS) {
    if (value < NOVAK_CHUNK_MIN || value > NOVAK_CHUNK_MAX || (value & (value - 1))) return fail(h, NOVAK_ERR_INVALID_ARG, "chunk_elems must be a power of two in [4096, 2^24]");
    if (value == h->chunk_elems) return NOVAK_OK;
    DeviceScope scope;
    NOVAK_HIP(h, scope.enter(h->device_id));
    // the old table may still be read by kernels in flight
    NOVAK_HIP(h, hipDeviceSynchronize());
    const int64_t old = h->chunk_elems;
    h->chunk_elems = value;
    const int rc = build_chunk_table(h);
    if (rc != NOVAK_OK) h->chunk_elems = old;
    return rc;
  }
  return fail(h, NOVAK_ERR_INVALID_ARG, "unknown tuning key");
}

int novak_set_tuning(novak_handle *h, int32_t key, int64_t value) {
  return guarded([&] { return set_tuning_impl(h, key, value); });
}

static int lookahead_init_impl(novak_handle *h, void *hip_stream) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (h->broken) return fail(h, NOVAK_ERR_STATE, "the handle lost its tables in a failed novak_set_tuning; destroy it");
  if (h->hp.lookahead_mode == NOVAK_LOOKAHEAD_NONE) return fail(h, NOVAK_ERR_STATE, "lookahead is off");
  if (h->n_chunks == 0) return NOVAK_OK;
  DeviceScope scope;
  NOVAK_HIP(h, scope.enter(h->device_id));
  launch_la<LA_INIT>(h, static_cast<hipStream_t>(hip_stream), tables_of(h), 0.0f, 0.0f);
  NOVAK_HIP(h, hipGetLastError());
  return NOVAK_OK;
}

static int step_impl(novak_handle *h, void *const *grads, int32_t grad_dtype, int64_t step, void *hip_stream) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (h->broken) return fail(h, NOVAK_ERR_STATE, "the handle lost its tables in a failed novak_set_tuning; destroy it");
  const size_t n = h->tensors.size();
  std::string why;
  int rc = check_grads(h->tensors.data(), n, grads, grad_dtype, &why);
  if (rc != NOVAK_OK) return fail(h, rc, why);
  const bool device_step = h->hp.device_step != 0;
  if (device_step) {
    if (step != 0) return fail(h, NOVAK_ERR_BAD_STEP, "in device-step mode the step count lives in device memory: pass step = 0");
    if (!h->d_counter) return fail(h, NOVAK_ERR_STATE, "device_step is on but novak_set_step_counter was not called");
  } else {
    if (step < 1) return fail(h, NOVAK_ERR_BAD_STEP, "step must be >= 1 (Eq. 5 is undefined at t = 0)");
    if (h->last_step != 0 && step != h->last_step + 1) return fail(h, NOVAK_ERR_BAD_STEP, "step must be the previous step + 1");
  }
  if (h->sync_due) return fail(h, NOVAK_ERR_STATE, "a lookahead sync is due before the next step");
  if (h->hp.auto_lr && !h->d_ema) return fail(h, NOVAK_ERR_STATE, "auto_lr is on but novak_set_auto_lr_state was not called");

  StepPlan pl;
  if (!device_step) plan_step(h->hp, step, &pl);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (h->n_chunks > 0 || device_step) {         // (a list without elements still counts its steps on the device)
    DeviceScope scope;
    NOVAK_HIP(h, scope.enter(h->device_id));
    // gradient pointers: upload only when the list changed since the previous step
    if (h->n_chunks > 0 && (!h->grads_uploaded || std::memcmp(h->last_grads.data(), grads, n * sizeof(void *)) != 0)) {
      // (the upload goes through a pinned staging slot that later calls reuse: not something a graph may replay)
      hipStreamCaptureStatus up_cs = hipStreamCaptureStatusNone;
      if (stream && hipStreamIsCapturing(stream, &up_cs) != hipSuccess) (void)hipGetLastError();
      if (up_cs == hipStreamCaptureStatusActive)
        return fail(h, NOVAK_ERR_STATE, "the gradient-pointer list differs from the previous step's while the stream is being captured: "
                                        "take one step with this list before the capture and keep the list fixed");
      const int slot = h->ring_next;
      h->ring_next = (slot + 1) % novak_handle::kRing;
      if (h->ring_used[slot]) NOVAK_HIP(h, hipEventSynchronize(h->ring_ev[slot]));
      void **src = h->h_ring + static_cast<size_t>(slot) * n;
      std::memcpy(src, grads, n * sizeof(void *));
      void *dst = static_cast<char *>(h->d_ptrs) + 4 * n * sizeof(void *);
      NOVAK_HIP(h, hipMemcpyAsync(dst, src, n * sizeof(void *), hipMemcpyHostToDevice, stream));
      NOVAK_HIP(h, hipEventRecord(h->ring_ev[slot], stream));
      h->ring_used[slot] = true;
      std::memcpy(h->last_grads.data(), grads, n * sizeof(void *));
      h->grads_uploaded = true;
    }
    if (device_step) {
      // Which record this step reads.  Eagerly: slot 0, written by a prologue just before.  Under capture: the
      // first step of a capture writes kDeviceRing records ahead and the following ones take the next slots.
      hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
      unsigned long long capture_id = 0;
      if (stream && hipStreamGetCaptureInfo(stream, &cs, &capture_id) != hipSuccess) {
        (void)hipGetLastError();
        cs = hipStreamCaptureStatusNone;
      }
      int slot = 0, n_records = 1;
      if (cs == hipStreamCaptureStatusActive) {
        if (!h->dev_in_capture || h->dev_capture_id != capture_id || h->dev_slot >= kDeviceRing) {
          h->dev_in_capture = true;
          h->dev_capture_id = capture_id;
          h->dev_slot = 0;
          n_records = kDeviceRing;
        } else {
          n_records = 0;
        }
        slot = h->dev_slot++;
      } else {
        h->dev_in_capture = false;
      }
      h->d_step = h->d_ring + slot;
      NOVAK_HIP(h, enqueue_step_device(h, grad_dtype, stream, n_records));
    } else {
      NOVAK_HIP(h, enqueue_step(h, grad_dtype, pl, stream));
    }
  }
  if (device_step) return NOVAK_OK;          // t is the device's business
  h->last_step = step;
  h->sync_due = (pl.window_closes && !h->hp.auto_sync) ? 1 : 0;
  return NOVAK_OK;
}

static int lookahead_sync_impl(novak_handle *h, void *hip_stream) {
  if (!h) return NOVAK_ERR_NULL_POINTER;
  if (h->broken) return fail(h, NOVAK_ERR_STATE, "the handle lost its tables in a failed novak_set_tuning; destroy it");
  if (h->hp.lookahead_mode == NOVAK_LOOKAHEAD_NONE) return fail(h, NOVAK_ERR_STATE, "lookahead is off");
  if (!h->sync_due) return fail(h, NOVAK_ERR_STATE, "no lookahead sync is due (sync follows the steps with t mod k == 0)");
  DeviceScope scope;
  NOVAK_HIP(h, scope.enter(h->device_id));
  NOVAK_HIP(h, launch_sync(h, static_cast<hipStream_t>(hip_stream)));
  h->sync_due = 0;
  return NOVAK_OK;
}

// Carves the static scratch array into the regions one call needs; false if they do not fit.
namespace {
struct StaticLayout {
  size_t chunks, ptrs, first_chunk, tensor_sums, scale, gscale, chunk_sums, end;
};
size_t align256(size_t x) { return (x + 255u) & ~size_t{255u}; }
StaticLayout static_layout(size_t n_tensors, size_t n_chunks, bool clip) {
  StaticLayout L;
  size_t o = 0;
  L.chunks = o;       o = align256(o + n_chunks * sizeof(novak_chunk));
  L.ptrs = o;         o = align256(o + n_tensors * (sizeof(TensorPtrs) + sizeof(void *)));
  L.first_chunk = o;  o = align256(o + (n_tensors + 1) * sizeof(int));
  L.tensor_sums = L.scale = L.gscale = L.chunk_sums = o;
  if (clip) {
    L.tensor_sums = o; o = align256(o + n_tensors * sizeof(NormSums));
    L.scale = o;       o = align256(o + n_tensors * sizeof(float));
    L.gscale = o;      o = align256(o + sizeof(float));
    L.chunk_sums = o;  o = align256(o + n_chunks * sizeof(NormSums));
  }
  L.end = o;
  return L;
}
}  // namespace

static int step_static_impl(const novak_hparams *hp, const novak_tensor_desc *tensors, int32_t n_tensors, void *const *grads,
                            int32_t grad_dtype, int64_t step, int32_t device_id, void *hip_stream) {
  if (!hp) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "hp is NULL");
  if (n_tensors < 0) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "n_tensors < 0");
  if (n_tensors > 0 && !tensors) return fail(nullptr, NOVAK_ERR_NULL_POINTER, "tensors is NULL");
  if (device_id < 0 || device_id >= kMaxDevices) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "device_id out of range");
  LaunchCtx cx;
  uint32_t warn = 0;
  int rc = novak_validate_hparams(hp, &cx.hp, &warn);
  if (rc != NOVAK_OK) return fail(nullptr, rc, "hyper-parameters rejected (section 5.8 validation rules)");
  if (scaled(&cx) || cx.hp.use_gc)
    return fail(nullptr, NOVAK_ERR_NOT_IMPLEMENTED, "the allocation-free step covers the single-pass update (with clipping and the sparse threshold); "
                                                    "layer adaptation, auto-LR and gradient centralization need a handle");
  if (cx.hp.device_step) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "the allocation-free step takes t as an argument: device_step must be 0");
  if (cx.hp.lookahead_mode != NOVAK_LOOKAHEAD_NONE && !cx.hp.auto_sync)
    return fail(nullptr, NOVAK_ERR_INVALID_ARG, "with lookahead on, the allocation-free step needs auto_sync = 1 (there is no handle to remember a due sync)");
  std::string why;
  rc = check_descs(cx.hp, tensors, n_tensors, &why);
  if (rc != NOVAK_OK) return fail(nullptr, rc, why);
  rc = check_grads(tensors, static_cast<size_t>(n_tensors), grads, grad_dtype, &why);
  if (rc != NOVAK_OK) return fail(nullptr, rc, why);
  if (step < 1) return fail(nullptr, NOVAK_ERR_BAD_STEP, "step must be >= 1 (Eq. 5 is undefined at t = 0)");
  if (n_tensors > NOVAK_STATIC_MAX_TENSORS) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "more than NOVAK_STATIC_MAX_TENSORS tensors");
  cx.chunk_elems = initial_chunk_elems(tensors, n_tensors, clipping(&cx), device_id, NOVAK_STATIC_MAX_CHUNKS);
  int64_t n_chunks = 0;
  for (int32_t i = 0; i < n_tensors; ++i) {
    n_chunks += (tensors[i].numel + cx.chunk_elems - 1) / cx.chunk_elems;
    if (n_chunks > NOVAK_STATIC_MAX_CHUNKS)
      return fail(nullptr, NOVAK_ERR_INVALID_ARG, "the list needs more than NOVAK_STATIC_MAX_CHUNKS chunk-table entries");
  }
  StepPlan pl;
  plan_step(cx.hp, step, &pl);
  if (n_chunks == 0) return NOVAK_OK;

  const StaticLayout L = static_layout(static_cast<size_t>(n_tensors), static_cast<size_t>(n_chunks), clipping(&cx));
  if (L.end > NOVAK_STATIC_SCRATCH_BYTES) return fail(nullptr, NOVAK_ERR_INVALID_ARG, "the tables do not fit the static scratch array");
  DeviceScope scope;
  NOVAK_HIP(nullptr, scope.enter(device_id));
  unsigned char *base = nullptr;
  NOVAK_HIP(nullptr, scratch_of(device_id, &base));
  int lds_cu = 0;
  if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device_id) == hipSuccess && lds_cu >= 65536)
    cx.lds_per_cu = lds_cu;
  cx.n_tensors = n_tensors;
  cx.n_chunks = n_chunks;
  cx.d_chunks = reinterpret_cast<novak_chunk *>(base + L.chunks);
  cx.d_ptrs = base + L.ptrs;
  cx.d_first_chunk = reinterpret_cast<int *>(base + L.first_chunk);
  if (clipping(&cx)) {
    cx.d_tensor_sums = reinterpret_cast<NormSums *>(base + L.tensor_sums);
    cx.d_scale = reinterpret_cast<float *>(base + L.scale);
    cx.d_gscale = reinterpret_cast<float *>(base + L.gscale);
    cx.d_chunk_sums = reinterpret_cast<NormSums *>(base + L.chunk_sums);
  }
  // tables: written by a kernel from its arguments, kFillBatch tensors per launch, in stream order before the step
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  TensorPtrs *d_tensors = reinterpret_cast<TensorPtrs *>(cx.d_ptrs);
  const void **d_grad = reinterpret_cast<const void **>(static_cast<char *>(cx.d_ptrs) + static_cast<size_t>(n_tensors) * sizeof(TensorPtrs));
  int64_t next_chunk = 0;
  for (int32_t first = 0; first < n_tensors; first += kFillBatch) {
    FillBatch b;
    b.count = n_tensors - first < kFillBatch ? n_tensors - first : kFillBatch;
    b.first_tensor = first;
    b.n_tensors = n_tensors;
    b.n_chunks = static_cast<int32_t>(n_chunks);
    b.chunk_elems = cx.chunk_elems;
    for (int32_t j = 0; j < b.count; ++j) {
      const novak_tensor_desc &d = tensors[first + j];
      FillTensor &ft = b.t[j];
      ft.ptrs.param = static_cast<float *>(d.param);
      ft.ptrs.m = static_cast<float *>(d.exp_avg);
      ft.ptrs.v = static_cast<float *>(d.exp_avg_sq);
      ft.ptrs.la = static_cast<float *>(d.la_buf);
      ft.grad = grads[first + j];
      ft.numel = d.numel;
      ft.first_chunk = next_chunk;
      next_chunk += (d.numel + cx.chunk_elems - 1) / cx.chunk_elems;
    }
    hipLaunchKernelGGL(novak_fill_tables_kernel, dim3(static_cast<unsigned>(b.count)), dim3(64), 0, stream, b, cx.d_chunks, d_tensors, d_grad,
                       cx.d_first_chunk);
    NOVAK_HIP(nullptr, hipGetLastError());
  }
  NOVAK_HIP(nullptr, enqueue_step(&cx, grad_dtype, pl, stream));
  return NOVAK_OK;
}

int novak_step_static(const novak_hparams *hp, const novak_tensor_desc *tensors, int32_t n_tensors, void *const *grads,
                      int32_t grad_dtype, int64_t step, int32_t device_id, void *hip_stream) {
  return guarded([&] { return step_static_impl(hp, tensors, n_tensors, grads, grad_dtype, step, device_id, hip_stream); });
}

// The entry points whose bodies stand above as *_impl.
int novak_arena_alloc(int32_t device_id, size_t bytes, void **ptr, int32_t *contiguous) {
  return guarded([&] { return arena_alloc_impl(device_id, bytes, ptr, contiguous); });
}

int novak_arena_free(int32_t device_id, void *ptr) {
  return guarded([&] { return arena_free_impl(device_id, ptr); });
}

int novak_nesterov_extrapolate(novak_handle *h, void *const *out, void *hip_stream) {
  return guarded([&] { return nesterov_extrapolate_impl(h, out, hip_stream); });
}

int novak_set_auto_lr_state(novak_handle *h, void *ema) {
  return guarded([&] { return set_auto_lr_state_impl(h, ema); });
}

int novak_set_step_counter(novak_handle *h, void *counter) {
  return guarded([&] { return set_step_counter_impl(h, counter); });
}

int novak_copy_tensor_scales(novak_handle *h, float *out, void *hip_stream) {
  return guarded([&] { return copy_tensor_scales_impl(h, out, hip_stream); });
}

int novak_lookahead_init(novak_handle *h, void *hip_stream) {
  return guarded([&] { return lookahead_init_impl(h, hip_stream); });
}

int novak_step(novak_handle *h, void *const *grads, int32_t grad_dtype, int64_t step, void *hip_stream) {
  return guarded([&] { return step_impl(h, grads, grad_dtype, step, hip_stream); });
}

int novak_lookahead_sync(novak_handle *h, void *hip_stream) {
  return guarded([&] { return lookahead_sync_impl(h, hip_stream); });
}

}  // extern "C"
