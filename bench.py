#!/usr/bin/env python3
"""Benchmark of the NOVAK update step on one MI355X.

A "step" is one pass of the whole hot path over the workload's parameter list: the scalar prologue,
the fused update kernel (with the lookahead accumulation) and, every k-th step, the slow-weight
synchronisation.  All tensors are resident in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Prints ONE JSON line: Gparams/s over the timed region, the roofline of the dominant kernel (HBM
bound; algorithmic bytes / HIP-event kernel time against 8 TB/s) and the CPU oracle's throughput on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5_decoder_1p3b")
    ap.add_argument("--lookahead", default=None, help="override: none | memory_efficient | basic")
    ap.add_argument("--nesterov", default=None, help="override: none | approx | classical | true")
    ap.add_argument("--la-k", type=int, default=None)
    ap.add_argument("--separate-sync", action="store_true", help="call novak_lookahead_sync instead of fusing the sync")
    ap.add_argument("--extrapolate", action="store_true",
                    help="true Nesterov: call novak_nesterov_extrapolate (Eq. 10) before every step, as a caller that evaluates the "
                         "gradient at the extrapolated point would; timed as its own kernel line")
    ap.add_argument("--layer-adaptation", action="store_true", help="research mode: per-tensor trust ratio (two-pass step)")
    ap.add_argument("--auto-lr", action="store_true", help="research mode: auto-LR factor (two-pass step)")
    ap.add_argument("--use-gc", action="store_true", help="research mode: gradient centralization of the multi-dimensional tensors")
    ap.add_argument("--clip", type=float, default=0.0, help="global-norm gradient clipping threshold (0 = off)")
    ap.add_argument("--sparse", type=float, default=0.0, help="sparse threshold tau of Eq. 27 (0 = off)")
    ap.add_argument("--grad-dtype", default=None, choices=("f32", "bf16"), help="override the workload's gradient type")
    ap.add_argument("--adaptive-beta", action="store_true", help="beta schedule of Eq. 3-4 (tau = 1000, 5000)")
    ap.add_argument("--moment-dtype", default="f32", choices=("f32", "bf16_m"),
                    help="storage of the first moment: fp32, or bfloat16 (reduced-precision state; not the headline configuration)")
    ap.add_argument("--layout", default="arena", choices=("arena", "torch_one", "separate", "separate_contiguous", "torch_pool"),
                    help="arena: one allocation from the library for all roles with a fixed spacing; torch_one: the same spacing "
                         "inside one ordinary torch allocation; separate: one torch allocation per role; separate_contiguous: one "
                         "novak_arena_alloc allocation per role; torch_pool: five separate torch allocations inside a torch.cuda.MemPool "
                         "whose segments come from the library (novak_torch_malloc)")
    ap.add_argument("--chunk-elems", type=int, default=None)
    ap.add_argument("--nontemporal", type=int, default=None)
    ap.add_argument("--vec-per-lane", type=int, default=None)
    ap.add_argument("--threads", type=int, default=None)
    ap.add_argument("--waves-per-cu", type=int, default=None)
    ap.add_argument("--prepass-waves-per-cu", type=int, default=None)
    ap.add_argument("--device-step", action="store_true",
                    help="device-step mode: the step count lives in device memory and a small kernel evaluates the scalar prologue")
    ap.add_argument("--graph-steps", type=int, default=0,
                    help="with --device-step: capture this many steps (a multiple of the lookahead window) into ONE HIP graph and time "
                         "its replays; --steps must be a multiple of it")
    ap.add_argument("--mode", default=None, choices=("fast", "research"), help="override the workload's dual-mode setting (section 7.1)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the comparison runs reported beside the headline (PyTorch-allocated layouts, separate sync kernel)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=1 << 22, help="elements of the oracle's timed sample")
    ap.add_argument("--cpu-workers", type=int, default=min(16, os.cpu_count() or 1),
                    help="processes of the all-cores oracle run reported beside the one-core cpu_baseline (<= 1: skip it)")
    return ap.parse_args()


def la_variant(lookahead: str, k: int, t: int, fused: bool) -> str:
    """Name of the step-kernel variant that step t runs (which lookahead stream it touches)."""
    if lookahead == "none":
        return "step"
    pos = (t - 1) % k + 1
    if lookahead == "memory_efficient":
        if pos == 1:
            return "step+la_first"
        if pos == k and fused:
            return "step+la_last_fused"
        return "step+la_mid"
    return "step+basic_fused" if (pos == k and fused) else "step"


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(workload: str, hyper, n_sample: int, budget_s: float = 12.0, max_steps: int = 200, seed: int = 42):
    """The oracle, as it stands, on n_sample elements shaped like the workload's largest tensor.

    Bounded: steps (with their syncs) are run until `budget_s` seconds of oracle time have been spent
    or `max_steps` steps are done; gradient generation is not timed.
    """
    import workloads as W
    from oracle import novak_oracle as O

    wl = W.get_workload(workload)
    n = min(n_sample, max(wl.numels))
    h = O.Hyper(**{k: v for k, v in hyper.items() if k not in ("mode", "auto_sync")})
    theta0 = W.host_params([n], seed)
    states = [O.init_state(theta0[0], h)]
    dt, steps = 0.0, 0
    while steps < max_steps and (dt < budget_s or (h.lookahead != "none" and steps % h.la_k != 0)):
        steps += 1
        g = W.host_grads([n], steps, wl.grad_std, seed, bf16=(wl.grad_dtype == "bf16"))[0]
        t0 = time.perf_counter()
        O.step(states[0], g, steps, h)
        if O.sync_due(steps, h):
            O.lookahead_sync(states[0], h)
        dt += time.perf_counter() - t0
    return {"value": n * steps / dt / 1e9, "unit": "Gparams/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n} elements of the largest tensor, {steps} steps incl. syncs, numpy fp64 arithmetic / "
                      f"fp32 state, {dt:.1f} s of oracle time", "host_cpus_visible": os.cpu_count(), "cpu_model": cpu_model()}


def _cpu_worker(job):
    return cpu_baseline(*job)


def cpu_baseline_all_cores(pool, workers: int, workload: str, hyper, n_sample: int):
    """The same oracle, unchanged, as `workers` independent processes, each on its own slice (a plain
    outer parallel-for over slices: the update is elementwise).  Reported beside the one-core figure."""
    parts = pool.map(_cpu_worker, [(workload, hyper, n_sample, 8.0, 200, 1000 + i) for i in range(workers)])
    return {"value": sum(p["value"] for p in parts), "unit": "Gparams/s", "cores": workers, "kind": "oracle",
            "sample": f"{workers} concurrent processes, each as in cpu_baseline with an 8 s budget on its own "
                      f"{n_sample}-element slice; sum of their rates"}


class Setup:
    """Device buffers of one workload in one layout, a library handle over them, and the timing loop.

    layout: "arena"  - one allocation from novak_arena_alloc (physically contiguous when the driver can),
                       roles placed by novak_plan_arena;
            "torch_one" - the same placement inside ONE ordinary torch allocation;
            "separate"  - five separate torch allocations (what a framework's optimizer usually holds).
    """

    def __init__(self, wl, hyper, layout, fused, args, torch, N, W):
        self.torch, self.N, self.wl, self.layout, self.fused = torch, N, wl, layout, fused
        dev = torch.device("cuda:0")
        numels = wl.numels
        self.p = wl.total
        rc, offsets, flat, stride = N.novak_plan_arena(numels)
        N.check(rc, "novak_plan_arena")
        flat = max(flat, 1)
        m_dtype = torch.bfloat16 if hyper["moment_dtype"] == "bf16_m" else torch.float32
        g_dtype = torch.bfloat16 if wl.grad_dtype == "bf16" else torch.float32
        self.arena_ptr, self.arena_contiguous, self.arena = None, 0, None
        self.role_ptrs, self.pool, self.views = [], None, None
        if layout == "separate_contiguous":
            torch.zeros(1, device=dev)
            views = []
            for i in range(5):      # each role its own physically contiguous allocation, bases 2 KB apart modulo 8 KB
                rc, ptr, contig = N.novak_arena_alloc(0, flat * 4 + 8192)
                N.check(rc, "novak_arena_alloc")
                self.role_ptrs.append(ptr)
                self.arena_contiguous = contig
                views.append(N.arena_as_tensor(ptr, flat * 4 + 8192, 0)[i * 2048:])
            self.views = views
        if layout == "arena":
            torch.zeros(1, device=dev)       # the device context exists before the library allocates on it
            rc, self.arena_ptr, self.arena_contiguous = N.novak_arena_alloc(0, 5 * stride)
            N.check(rc, "novak_arena_alloc")
            self.arena = N.arena_as_tensor(self.arena_ptr, 5 * stride, 0)
        elif layout == "torch_one":
            self.arena = torch.empty(5 * stride, dtype=torch.uint8, device=dev)
        if self.arena is not None:
            self.arena.zero_()
            arena = self.arena

            def role(i, dtype):
                return arena[i * stride: i * stride + flat * dtype.itemsize].view(dtype)
        elif layout == "separate_contiguous":
            def role(i, dtype):
                t = self.views[i][: flat * dtype.itemsize].view(dtype)
                t.zero_()
                return t
        elif layout == "torch_pool":
            self.pool = N.torch_mem_pool()

            def role(i, dtype):
                with torch.cuda.use_mem_pool(self.pool):
                    return torch.zeros(flat, dtype=dtype, device=dev)
        else:
            def role(i, dtype):
                return torch.zeros(flat, dtype=dtype, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(42)
        theta, m, v, la, grad = role(0, torch.float32), role(1, m_dtype), role(2, torch.float32), role(3, torch.float32), role(4, g_dtype)
        theta.normal_(0.0, W.PARAM_STD, generator=gen)
        g32 = torch.empty(flat, dtype=torch.float32, device=dev).normal_(0.0, wl.grad_std, generator=gen)
        grad.copy_(g32)          # rounds to nearest-even when the gradients are bfloat16
        del g32
        self.bufs = (theta, m, v, la, grad)

        self.device_step = bool(args.device_step)
        hp = N.make_hparams(auto_sync=fused, device_step=self.device_step, **hyper)
        descs = [N.novak_tensor_desc(theta.data_ptr() + 4 * o, m.data_ptr() + m.element_size() * o, v.data_ptr() + 4 * o,
                                     la.data_ptr() + 4 * o, n, r) for o, n, r in zip(offsets, numels, wl.rows)]
        rc, self.handle = N.novak_create(hp, descs, 0)
        N.check(rc, "novak_create")
        handle = self.handle
        for key, val in ((N.NOVAK_TUNE_CHUNK_ELEMS, args.chunk_elems), (N.NOVAK_TUNE_NONTEMPORAL, args.nontemporal),
                         (N.NOVAK_TUNE_VEC_PER_LANE, args.vec_per_lane), (N.NOVAK_TUNE_THREADS, args.threads),
                         (N.NOVAK_TUNE_WAVES_PER_CU, args.waves_per_cu), (N.NOVAK_TUNE_PREPASS_WAVES_PER_CU, args.prepass_waves_per_cu)):
            if val is not None:
                N.check(N.novak_set_tuning(handle, key, val), "set_tuning", handle)
        rc, self.info = N.novak_get_info(handle)
        info = self.info
        self.la_name = {0: "none", 1: "memory_efficient", 2: "basic"}[info.lookahead_mode]
        self.nest_name = {0: "none", 1: "approx", 2: "classical", 3: "true"}[info.nesterov_mode]
        self.k = int(hyper["la_k"])
        self.gdt = N.GRAD_DTYPE[wl.grad_dtype]
        self.grad_arr = (C.c_void_p * len(numels))(*[grad.data_ptr() + grad.element_size() * o for o in offsets])
        self.stream = torch.cuda.current_stream().cuda_stream
        if self.la_name != "none":
            N.check(N.novak_lookahead_init(handle, self.stream), "lookahead_init", handle)
        self.counter = torch.zeros(1, dtype=torch.int64, device=dev)
        if self.device_step:
            N.check(N.novak_set_step_counter(handle, self.counter.data_ptr()), "set_step_counter", handle)
        self.graph_steps = int(args.graph_steps) if self.device_step else 0
        self.ema = torch.zeros(2, dtype=torch.float64, device=dev)
        if info.auto_lr:
            N.check(N.novak_set_auto_lr_state(handle, self.ema.data_ptr()), "set_auto_lr_state", handle)
        self.extrapolate_arr = None
        if args.extrapolate:
            self.extra_out = torch.empty(flat, dtype=torch.float32, device=dev)
            self.extrapolate_arr = (C.c_void_p * len(numels))(*[self.extra_out.data_ptr() + 4 * o for o in offsets])
        # the trust ratio makes the step two-pass; auto-LR alone is the single-pass step behind a norms pre-pass
        self.scaled = bool(info.layer_adaptation)
        self.auto_only = bool(info.auto_lr and not info.layer_adaptation)
        self.m_tag = "+bf16_m" if info.moment_dtype == N.NOVAK_MOMENT_BF16_M else ""
        self.t = 0
        # extra gradient reads of the pre-pass (one read serves clipping and centralization; with centralization
        # alone only the centralized tensors are read)
        self.extra_bpp = 0.0
        if hyper["clip_threshold"] > 0 or self.auto_only:
            self.extra_bpp = N.novak_bytes_per_param_clip(self.gdt)
        elif info.use_gc:
            self.extra_bpp = N.novak_bytes_per_param_clip(self.gdt) * sum(n for n, r in zip(numels, wl.rows) if r >= 1) / max(self.p, 1)
        if self.auto_only:
            self.extra_bpp += 4.0        # the pre-pass over the parameters (fp32) for their global norm

    def one_step(self):
        N, handle = self.N, self.handle
        self.t += 1
        N.check(N.novak_step(handle, self.grad_arr, self.gdt, 0 if self.device_step else self.t, self.stream), "novak_step", handle)
        if self.la_name != "none" and not self.fused and self.t % self.k == 0:
            N.check(N.novak_lookahead_sync(handle, self.stream), "novak_lookahead_sync", handle)
            return True
        return False

    def timed_graph(self, warmup, steps):
        """Device-step mode: graph_steps steps captured into ONE HIP graph (through torch's stream capture), replayed
        steps / graph_steps times; every replay continues from the device's own step counter."""
        torch, N, g = self.torch, self.N, self.graph_steps
        if steps % g or (self.la_name != "none" and g % self.k):
            raise SystemExit("bench.py: --steps must be a multiple of --graph-steps, and that of the lookahead window")
        for _ in range(max(warmup, 1) + (-max(warmup, 1)) % (self.k if self.la_name != "none" else 1)):
            self.one_step()               # eager: uploads the gradient-pointer list; ends on a window boundary
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cap_stream = torch.cuda.current_stream().cuda_stream
            for _ in range(g):
                N.check(N.novak_step(self.handle, self.grad_arr, self.gdt, 0, cap_stream), "novak_step (capture)", self.handle)
        replays = steps // g
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for a, b in ev:
            a.record()
            graph.replay()
            b.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_begin
        expect = self.t + steps
        assert int(self.counter.item()) == expect, "the replays did not advance the device's step counter"
        names = [("scaled_" if self.scaled else "") + la_variant(self.la_name, self.k, self.t + 1 + i, self.fused) + self.m_tag for i in range(g)]
        self.t = expect
        bpp = sum(self.bytes_of(n) for n in names)
        ms = [a.elapsed_time(b) for a, b in ev]
        avg = sum(ms) / len(ms)
        name = f"graph_of_{g}_steps"
        kernels = {name: {"launches": replays, "avg_ms": avg, "bytes_per_param": bpp, "GBps": self.p * bpp / (avg * 1e-3) / 1e9,
                          "avg_ms_per_step": avg / g}}
        del graph
        return {"elapsed": elapsed, "value": self.p * steps / elapsed / 1e9, "ms_per_step": elapsed / steps * 1e3,
                "kernels": kernels, "dominant": name}

    def bytes_of(self, name):
        """Algorithmic bytes per parameter of a step variant (a two-pass "scaled_" step is timed as a whole)."""
        N, info, k = self.N, self.info, self.k
        two = name.startswith("scaled_")
        fn = N.novak_bytes_per_param_scaled_step if two else N.novak_bytes_per_param_step
        base = name[len("scaled_"):] if two else name
        base = base[:len(base) - len(self.m_tag)] if self.m_tag else base
        pos = {"step": 2 if self.la_name == "basic" else 1, "step+la_first": 1, "step+la_mid": 2,
               "step+la_last_fused": k, "step+basic_fused": k}[base]
        saved = N.novak_bytes_per_param_moment_saving(info.moment_dtype, int(two))
        la_mode = info.lookahead_mode
        return self.extra_bpp - saved + (fn(la_mode, self.gdt, k, pos, int(self.fused)) if self.la_name != "none" else fn(0, self.gdt, k, 1, 0))

    def timed(self, warmup, steps):
        """W untimed steps, then exactly K steps between synchronisations, each bracketed by HIP events on the launch stream."""
        torch, N = self.torch, self.N
        if self.graph_steps:
            return self.timed_graph(warmup, steps)
        for _ in range(warmup):
            if self.extrapolate_arr is not None:
                N.check(N.novak_nesterov_extrapolate(self.handle, self.extrapolate_arr, self.stream), "novak_nesterov_extrapolate", self.handle)
            self.one_step()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        variants, sync_ev, extra_ev = [], [], []
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(steps):
            variants.append(("scaled_" if self.scaled else "") + la_variant(self.la_name, self.k, self.t + 1, self.fused) + self.m_tag)
            if self.extrapolate_arr is not None:
                x0 = torch.cuda.Event(enable_timing=True)
                x0.record()
                N.check(N.novak_nesterov_extrapolate(self.handle, self.extrapolate_arr, self.stream), "novak_nesterov_extrapolate", self.handle)
                extra_ev.append((x0, ev[i][0]))
            ev[i][0].record()
            self.t += 1
            N.check(N.novak_step(self.handle, self.grad_arr, self.gdt, 0 if self.device_step else self.t, self.stream), "novak_step", self.handle)
            ev[i][1].record()
            if self.la_name != "none" and not self.fused and self.t % self.k == 0:
                N.check(N.novak_lookahead_sync(self.handle, self.stream), "novak_lookahead_sync", self.handle)
                done = torch.cuda.Event(enable_timing=True)
                done.record()
                sync_ev.append((ev[i][1], done))
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_begin
        per = {}
        for name, (a, b) in zip(variants, ev):
            per.setdefault(name, []).append(a.elapsed_time(b))     # ms
        p = self.p
        kernels = {}
        for name, ms in per.items():
            avg, bpp = sum(ms) / len(ms), self.bytes_of(name)
            kernels[name] = {"launches": len(ms), "avg_ms": avg, "bytes_per_param": bpp, "GBps": p * bpp / (avg * 1e-3) / 1e9}
        if sync_ev:     # the separate slow-weight synchronisation kernel (Eq. 30-31), timed from the end of its step
            ms = [a.elapsed_time(b) for a, b in sync_ev]
            avg, bpp = sum(ms) / len(ms), N.novak_bytes_per_param_sync(self.info.lookahead_mode)
            kernels["lookahead_sync"] = {"launches": len(ms), "avg_ms": avg, "bytes_per_param": bpp, "GBps": p * bpp / (avg * 1e-3) / 1e9}
        if extra_ev:    # Eq. 10: theta and m read, the extrapolated point written
            ms = [a.elapsed_time(b) for a, b in extra_ev]
            avg, bpp = sum(ms) / len(ms), 12.0 - (2.0 if self.m_tag else 0.0)
            kernels["nesterov_extrapolate"] = {"launches": len(ms), "avg_ms": avg, "bytes_per_param": bpp, "GBps": p * bpp / (avg * 1e-3) / 1e9}
        dominant = max(kernels, key=lambda n: kernels[n]["launches"] * kernels[n]["avg_ms"])
        return {"elapsed": elapsed, "value": p * steps / elapsed / 1e9, "ms_per_step": elapsed / steps * 1e3,
                "kernels": kernels, "dominant": dominant}

    def close(self):
        self.torch.cuda.synchronize()
        self.N.novak_destroy(self.handle)
        self.bufs = None
        if self.arena_ptr is not None:
            self.arena = None
            self.N.check(self.N.novak_arena_free(0, self.arena_ptr), "novak_arena_free")
        self.arena = None
        self.pool = None
        self.views = None
        for ptr in self.role_ptrs:
            self.N.check(self.N.novak_arena_free(0, ptr), "novak_arena_free")
        self.role_ptrs = []
        self.torch.cuda.empty_cache()


def brief(r):
    """The figures of a comparison run that go beside the headline."""
    k = r["kernels"][r["dominant"]]
    return {"value": r["value"], "unit": "Gparams/s", "ms_per_step": r["ms_per_step"], "dominant_kernel": r["dominant"],
            "GBps": k["GBps"], "frac": k["GBps"] / HBM_PEAK_GBS}


def main():
    args = parse_args()
    pool, workers = None, 0
    if args.gpus == 1 and not args.no_cpu_baseline and args.cpu_workers > 1:
        # started before anything touches the GPU; the workers idle until the GPU part is over
        import multiprocessing as mp
        workers = args.cpu_workers
        pool = mp.get_context("spawn").Pool(workers)
    from paper_2601_07876_amd import build as B
    B.ensure_built()                 # loads what was built beforehand; builds only where nothing is there
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the update is elementwise and would shard "
              "without communication)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    from paper_2601_07876_amd import novak as N

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(torch.device("cuda:0"))

    wl = W.get_workload(args.workload)
    if args.grad_dtype:
        wl = dataclasses.replace(wl, grad_dtype=args.grad_dtype)
    hyper = dict(wl.hyper)
    if args.lookahead:
        hyper["lookahead"] = args.lookahead
    if args.nesterov:
        hyper["nesterov"] = args.nesterov
    if args.la_k:
        hyper["la_k"] = args.la_k
    if args.mode:
        hyper["mode"] = args.mode
    if args.layer_adaptation or args.auto_lr or args.use_gc:
        hyper.update(mode="research", layer_adaptation=args.layer_adaptation, auto_lr=args.auto_lr, use_gc=args.use_gc)
    hyper.update(clip_threshold=args.clip, sparse_threshold=args.sparse, moment_dtype=args.moment_dtype)
    if args.adaptive_beta:
        hyper.update(adaptive_beta=True)
    fused = not args.separate_sync
    p = wl.total

    # ---- the headline: the requested layout (default: the library's arena) and sync mode (default: fused) ----
    run = Setup(wl, hyper, args.layout, fused, args, torch, N, W)
    info, la_name, nest_name, k = run.info, run.la_name, run.nest_name, run.k
    arena_contiguous = run.arena_contiguous
    res = run.timed(args.warmup, args.steps)
    run.close()
    kernels, dominant = res["kernels"], res["dominant"]
    dk = kernels[dominant]
    running = profiled_config_of(args, fused, int(info.chunk_elems))
    traffic, traffic_file = measured_traffic(args.workload, dominant, running)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": dk["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dk["GBps"] / HBM_PEAK_GBS, "avg_kernel_ms": dk["avg_ms"],
                "algorithmic_bytes_per_launch": p * dk["bytes_per_param"], "traffic": traffic}
    if traffic:
        # counters come from a separate rocprofv3 --pmc run of this same configuration, committed under profiles/
        roofline["traffic_source"] = traffic_file
        roofline["traffic_over_algorithmic"] = traffic / (p * dk["bytes_per_param"])

    result = {
        "metric": "Gparams updated/s per NOVAK step",
        "value": res["value"],
        "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "params": p, "tensors": len(wl.numels), "grad_dtype": wl.grad_dtype,
                   "nesterov": nest_name, "lookahead": la_name, "la_k": k, "sync": "fused" if fused else "separate",
                   "mode": hyper["mode"], "rectified": bool(hyper["rectified"]),
                   "layer_adaptation": bool(info.layer_adaptation), "auto_lr": bool(info.auto_lr),
                   "use_gc": bool(info.use_gc), "moment_dtype": args.moment_dtype, "clip_threshold": args.clip, "sparse_threshold": args.sparse, "adaptive_beta": bool(args.adaptive_beta),
                   "step_count": "device" if args.device_step else "host", "graph_steps": int(args.graph_steps) if args.device_step else 0,
                   "chunk_elems": int(info.chunk_elems), "chunks": int(info.n_chunks), "layout": args.layout,
                   "arena_contiguous": bool(arena_contiguous)},
        "roofline": roofline,
        "kernels": kernels,
    }

    # ---- beside it, in the same process: what a caller gets whose memory comes from PyTorch, and the sync as a
    # ---- separate kernel (the benchmark spec names both); skipped when a specific layout / sync mode was asked for
    if not args.no_extras and args.layout == "arena" and fused and not args.device_step:
        others = {}
        for name, layout in (("torch_one_allocation_planned_layout", "torch_one"), ("torch_five_separate_allocations", "separate"),
                             ("torch_five_allocations_in_a_mem_pool_fed_by_the_library", "torch_pool")):
            try:
                r2 = Setup(wl, hyper, layout, True, args, torch, N, W)
            except (RuntimeError, AttributeError) as e:      # a torch build without MemPool / pluggable allocators
                if layout != "torch_pool":
                    raise
                others[name] = {"unavailable": str(e)[:200]}
                continue
            others[name] = brief(r2.timed(args.warmup, args.steps))
            r2.close()
        result["other_layouts"] = others
        if la_name != "none":
            r3 = Setup(wl, hyper, "arena", False, args, torch, N, W)
            t3 = r3.timed(args.warmup, args.steps)
            r3.close()
            sk = t3["kernels"].get("lookahead_sync")
            result["separate_sync"] = {"value": t3["value"], "unit": "Gparams/s", "ms_per_step": t3["ms_per_step"],
                                       "note": "novak_lookahead_sync as its own kernel after every k-th step, amortised over the timed steps",
                                       "sync_kernel": ({**sk, "frac": sk["GBps"] / HBM_PEAK_GBS} if sk else None)}

    if not args.no_cpu_baseline:
        eff = {**hyper, "nesterov": nest_name, "lookahead": la_name, "layer_adaptation": bool(info.layer_adaptation),
               "auto_lr": bool(info.auto_lr), "use_gc": False}
        result["cpu_baseline"] = cpu_baseline(wl.name, eff, args.cpu_sample)
        if pool is not None:
            result["cpu_baseline_all_cores"] = cpu_baseline_all_cores(pool, workers, wl.name, eff, args.cpu_sample)
            pool.close()
            pool.join()
    print(json.dumps(result))


def profiled_config_of(args, fused, chunk_elems: int) -> str:
    """The launch configuration as the profiles/ summaries state it (a counter figure is only carried over
    to a run of the same configuration)."""
    auto = lambda x, d: d if x is None else x
    if args.device_step:
        return "device_step"          # another kernel variant than the one the counters were taken on
    return (f"layout={args.layout} chunk_elems={chunk_elems} waves_per_cu={auto(args.waves_per_cu, 0)} "
            f"nontemporal={auto(args.nontemporal, 1)} vec_per_lane={auto(args.vec_per_lane, 1)} threads={auto(args.threads, 64)} "
            f"sync={'fused' if fused else 'separate'}")


def measured_traffic(workload: str, kernel: str, running_config: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this workload
    (profiles/traffic_*.txt), if that summary was taken in the running launch configuration; else (None, None)."""
    name = f"traffic_{workload}.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    lines = open(path).read().splitlines()
    if not any(l.strip() == "profiled_config " + running_config for l in lines):
        return None, None
    for line in lines:
        parts = line.split()
        if len(parts) >= 3 and parts[0] == "hbm_bytes_per_launch" and parts[1] == kernel:
            return float(parts[2]), "profiles/" + name
    return None, None


if __name__ == "__main__":
    main()
