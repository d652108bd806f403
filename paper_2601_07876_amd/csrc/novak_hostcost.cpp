// novak_hostcost: how long the library itself keeps the host busy per novak_step, without Python in the way.
//
//   novak_hostcost NUMELS_FILE [STEPS [GRAPH_STEPS [WAVES_PER_CU]]]
//
// NUMELS_FILE lists one tensor size per line (the shape lists of the benchmark workloads can be written with
// `python -c "import workloads as W; print(*W.get_workload('c2_resnet50').numels, sep='\n')"`).  The tensors
// are placed in five device arrays as novak_plan_arena recommends; values are zero (the host path does not
// depend on them).  The default hyper-parameters are the workloads' (rectified, Nesterov approximation,
// memory-efficient lookahead k = 5 fused into the k-th step).
// Prints one JSON line: host_us_per_step = wall time of STEPS back-to-back novak_step calls divided by STEPS
// (validation, scalar prologue, launch; the calls return before the kernels run), and total_us_per_step =
// the same including the wait for the last kernel (what a step costs when the GPU is the bottleneck).
// With GRAPH_STEPS > 0 (a multiple of 5 that divides STEPS) the handle runs in device-step mode (step count in
// device memory) on a stream of its own: the same two figures for the eager loop, then GRAPH_STEPS steps are
// captured once into a HIP graph and replayed STEPS / GRAPH_STEPS times: graph_us_per_step.
// WAVES_PER_CU > 0 overrides the residency cap of the step kernels (NOVAK_TUNE_WAVES_PER_CU).
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "novak.h"

#define CK(call)                                                                      \
  do {                                                                                \
    hipError_t e_ = (call);                                                           \
    if (e_ != hipSuccess) {                                                           \
      std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                 \
      return 1;                                                                       \
    }                                                                                 \
  } while (0)
#define NK(call)                                                                                      \
  do {                                                                                                \
    int rc_ = (call);                                                                                 \
    if (rc_ != NOVAK_OK) {                                                                            \
      std::fprintf(stderr, "%s: %s (%s)\n", #call, novak_status_string(rc_), novak_last_error(h));    \
      return 1;                                                                                       \
    }                                                                                                 \
  } while (0)

int main(int argc, char **argv) {
  if (argc < 2) {
    std::fprintf(stderr, "usage: %s NUMELS_FILE [STEPS [GRAPH_STEPS [WAVES_PER_CU]]]\n", argv[0]);
    return 2;
  }
  const int steps = argc > 2 ? std::atoi(argv[2]) : 2000;
  const int graph_steps = argc > 3 ? std::atoi(argv[3]) : 0;
  const int waves_per_cu = argc > 4 ? std::atoi(argv[4]) : 0;
  if (graph_steps < 0 || (graph_steps > 0 && (graph_steps % 5 != 0 || steps % graph_steps != 0))) {
    std::fprintf(stderr, "GRAPH_STEPS must be a multiple of the lookahead window (5) that divides STEPS\n");
    return 2;
  }
  std::vector<int64_t> numels;
  {
    std::FILE *f = std::fopen(argv[1], "r");
    if (!f) { std::perror(argv[1]); return 2; }
    long long x;
    while (std::fscanf(f, "%lld", &x) == 1) numels.push_back(x);
    std::fclose(f);
  }
  const int32_t n = static_cast<int32_t>(numels.size());
  if (n == 0 || steps < 1) { std::fprintf(stderr, "nothing to do\n"); return 2; }
  novak_handle *h = nullptr;
  std::vector<int64_t> offs(numels.size());
  int64_t role_elems = 0, stride = 0;
  NK(novak_plan_arena(numels.data(), n, offs.data(), &role_elems, &stride));
  char *arena = nullptr;
  CK(hipSetDevice(0));
  CK(hipMalloc(reinterpret_cast<void **>(&arena), static_cast<size_t>(5 * stride)));
  CK(hipMemset(arena, 0, static_cast<size_t>(5 * stride)));

  novak_hparams hp;
  std::memset(&hp, 0, sizeof hp);
  hp.struct_size = sizeof hp;
  hp.lr = 1e-3; hp.beta1 = 0.9; hp.beta2 = 0.999; hp.eps = 1e-8; hp.weight_decay = 1e-2; hp.beta_n = 0.9;
  hp.la_alpha = 0.5; hp.la_k = 5; hp.rectified = 1; hp.decoupled_decay = 1;
  hp.nesterov_mode = NOVAK_NESTEROV_APPROX; hp.lookahead_mode = NOVAK_LOOKAHEAD_MEMORY_EFFICIENT;
  hp.unrect_fallback = NOVAK_UNRECT_ADAM_DENOM; hp.mode = NOVAK_MODE_FAST; hp.auto_sync = 1;
  hp.auto_lr_gamma = 0.1; hp.trust_clip_lo = 0.1; hp.trust_clip_hi = 10.0; hp.auto_clip_lo = 0.1; hp.auto_clip_hi = 2.0;
  hp.beta_tau1 = 1000.0; hp.beta_tau2 = 5000.0;
  hp.device_step = graph_steps > 0 ? 1 : 0;
  std::vector<novak_tensor_desc> descs(numels.size());
  std::vector<void *> grads(numels.size());
  int64_t total = 0;
  for (int32_t i = 0; i < n; ++i) {
    char *base = arena + 4 * offs[static_cast<size_t>(i)];
    descs[static_cast<size_t>(i)] = novak_tensor_desc{base, base + stride, base + 2 * stride, base + 3 * stride, numels[static_cast<size_t>(i)], 0};
    grads[static_cast<size_t>(i)] = base + 4 * stride;
    total += numels[static_cast<size_t>(i)];
  }
  NK(novak_create(&h, &hp, descs.data(), n, 0));
  if (waves_per_cu > 0) NK(novak_set_tuning(h, NOVAK_TUNE_WAVES_PER_CU, waves_per_cu));
  hipStream_t stream = nullptr;                 // the legacy default stream cannot be captured
  int64_t *counter = nullptr;
  if (graph_steps > 0) {
    CK(hipStreamCreate(&stream));
    CK(hipMalloc(reinterpret_cast<void **>(&counter), sizeof(int64_t)));
    CK(hipMemset(counter, 0, sizeof(int64_t)));
    NK(novak_set_step_counter(h, counter));
  }
  NK(novak_lookahead_init(h, stream));
  int64_t t = 0;
  // in device-step mode the `step` argument is 0 and the device counts
  auto step_arg = [&]() -> int64_t { ++t; return graph_steps > 0 ? 0 : t; };
  for (int i = 0; i < 200; ++i) NK(novak_step(h, grads.data(), NOVAK_GRAD_F32, step_arg(), stream));
  CK(hipDeviceSynchronize());
  using clock = std::chrono::steady_clock;
  const auto t0 = clock::now();
  for (int i = 0; i < steps; ++i) NK(novak_step(h, grads.data(), NOVAK_GRAD_F32, step_arg(), stream));
  const auto t1 = clock::now();
  CK(hipDeviceSynchronize());
  const auto t2 = clock::now();
  const double host_us = std::chrono::duration<double, std::micro>(t1 - t0).count() / steps;
  const double total_us = std::chrono::duration<double, std::micro>(t2 - t0).count() / steps;
  std::printf("{\"tensors\": %d, \"params\": %lld, \"steps\": %d, \"step_count\": \"%s\", \"host_us_per_step\": %.3f, "
              "\"total_us_per_step\": %.3f, \"Gparams_per_s\": %.2f",
              n, static_cast<long long>(total), steps, graph_steps > 0 ? "device" : "host", host_us, total_us,
              static_cast<double>(total) / total_us / 1e3);
  if (graph_steps > 0) {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    CK(hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal));
    for (int i = 0; i < graph_steps; ++i) NK(novak_step(h, grads.data(), NOVAK_GRAD_F32, 0, stream));
    CK(hipStreamEndCapture(stream, &graph));
    CK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    const int replays = steps / graph_steps;
    for (int i = 0; i < 2; ++i) CK(hipGraphLaunch(exec, stream));          // warm-up
    CK(hipStreamSynchronize(stream));
    const auto g0 = clock::now();
    for (int i = 0; i < replays; ++i) CK(hipGraphLaunch(exec, stream));
    const auto g1 = clock::now();
    CK(hipStreamSynchronize(stream));
    const auto g2 = clock::now();
    int64_t counted = 0;
    CK(hipMemcpy(&counted, counter, sizeof counted, hipMemcpyDeviceToHost));
    const int64_t expect = 200 + steps + static_cast<int64_t>(2 + replays) * graph_steps;
    if (counted != expect) {
      std::fprintf(stderr, "the device counted %lld steps, expected %lld\n", static_cast<long long>(counted), static_cast<long long>(expect));
      return 1;
    }
    std::printf(", \"graph_steps\": %d, \"graph_host_us_per_step\": %.3f, \"graph_us_per_step\": %.3f, \"graph_Gparams_per_s\": %.2f",
                graph_steps, std::chrono::duration<double, std::micro>(g1 - g0).count() / steps,
                std::chrono::duration<double, std::micro>(g2 - g0).count() / steps,
                static_cast<double>(total) / (std::chrono::duration<double, std::micro>(g2 - g0).count() / steps) / 1e3);
    CK(hipGraphExecDestroy(exec));
    CK(hipGraphDestroy(graph));
  }
  std::printf("}\n");
  NK(novak_destroy(h));
  if (counter) CK(hipFree(counter));
  if (stream) CK(hipStreamDestroy(stream));
  CK(hipFree(arena));
  return 0;
}
