"""GPU parity at the full benchmark sizes (C2..C5), in the launch configuration bench.py times.

Inputs are drawn on the device from a seeded torch generator (input plumbing, not the method); the
oracle receives copies of the sampled elements' inputs and computes those elements one by one (the
update is elementwise, so a sample of elements is a valid run).  Samples always include tensor
heads and tails and elements on both sides of chunk-table boundaries.  Every sampled element of
theta, m, v (and the lookahead buffer where it is defined) must meet |gpu - ref| <= 1e-7 + 1e-5|ref|.
Two runs give the oracle EVERY element instead of a sample: the whole ResNet-50 list, and one whole
8192 x 2048 tensor inside the 1.3B list, both in the arena layout bench.py times.
On top of that, whole-buffer properties that hold at any size are checked: v >= 0, finiteness,
and that elements outside every tensor (guard gaps between tensors) are untouched.
Runs with a bfloat16 first moment are compared after every step from a common state (tests/harness.py).
"""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N
from tests import harness as H

pytestmark = pytest.mark.gpu

GAP = 64          # guard elements between consecutive tensors in the flat buffers (keeps 256-B alignment)
SENTINEL = 768.0      # exactly representable in bfloat16 too


def _say(msg):
    print(msg, flush=True)


class FullRun:
    """Flat device buffers holding a whole workload, a library handle, and the sampled oracle."""

    def __init__(self, wl: W.Workload, samples_per_tensor: int = 2048, seed: int = 42, device="cuda:0", arena: bool = False,
                 dense=()):
        """arena=True places all five roles in ONE allocation as novak_plan_arena recommends (the layout
        bench.py times); otherwise every role is its own allocation with GAP guard elements around each tensor.
        `dense`: indices of tensors of which EVERY element goes to the oracle ("all" = the whole list)."""
        self.wl, self.seed = wl, seed
        self.dev = torch.device(device)
        self.numels = wl.numels
        self.arena = None
        if arena:
            rc, self.offsets, self.flat_len, self.stride = N.novak_plan_arena(self.numels)
            N.check(rc, "novak_plan_arena")
            torch.zeros(1, device=self.dev)
            rc, self.arena_ptr, self.arena_contiguous = N.novak_arena_alloc(0, 5 * self.stride)
            N.check(rc, "novak_arena_alloc")
            self.arena = N.arena_as_tensor(self.arena_ptr, 5 * self.stride, 0)
            self.ends = self.offsets[1:] + [self.flat_len]          # padding after a tensor runs up to the next one
        else:
            self.offsets = []
            off = GAP
            for n in self.numels:
                self.offsets.append(off)
                off += ((n + GAP - 1) // GAP) * GAP + GAP
            self.flat_len = off
        gdt = torch.bfloat16 if wl.grad_dtype == "bf16" else torch.float32
        self.bufs = {r: self._role(i, torch.float32) for i, r in enumerate(("theta", "m", "v", "la"))}
        self.g = self._role(4, gdt)
        self.gen = torch.Generator(device=self.dev)
        self.chunk_elems = None
        self.handle = None
        # sampled global indices
        idx = []
        for i, n in enumerate(self.numels):
            if dense == "all" or i in dense:
                idx.append(np.arange(n, dtype=np.int64) + self.offsets[i])
            else:
                idx.append(W.sample_indices(n, samples_per_tensor, seed, i, block=16384) + self.offsets[i])
        self.idx_host = np.concatenate(idx)
        self.idx = torch.from_numpy(self.idx_host).to(self.dev)
        # every position of the flat buffers that belongs to no tensor (guard gaps, alignment padding)
        gaps, end = [], 0
        for o, n in zip(self.offsets, self.numels):
            gaps.append(np.arange(end, o, dtype=np.int64))
            end = o + n
        gaps.append(np.arange(end, self.flat_len, dtype=np.int64))
        self.outside = torch.from_numpy(np.concatenate(gaps)).to(self.dev)
        self._grad_arr = (C.c_void_p * len(self.numels))()
        for i, (o, n) in enumerate(zip(self.offsets, self.numels)):
            self._grad_arr[i] = self.g.data_ptr() + o * self.g.element_size()

    def _role(self, i, dtype):
        if self.arena is None:
            return torch.empty(self.flat_len, dtype=dtype, device=self.dev)
        return self.arena[i * self.stride: i * self.stride + self.flat_len * dtype.itemsize].view(dtype)

    def reset(self, hyper, auto_sync=False):
        if self.handle is not None:
            torch.cuda.synchronize()
            N.novak_destroy(self.handle)
        self.gen.manual_seed(self.seed)
        self.bf16_m = hyper.get("moment_dtype", "f32") == "bf16_m"
        want = torch.bfloat16 if self.bf16_m else torch.float32
        if self.bufs["m"].dtype != want:
            del self.bufs["m"]
            self.bufs["m"] = self._role(1, want)
        for r in ("theta", "m", "v", "la"):
            self.bufs[r].fill_(SENTINEL)
        for o, n in zip(self.offsets, self.numels):
            self.bufs["theta"][o:o + n].normal_(0.0, W.PARAM_STD, generator=self.gen)
            self.bufs["m"][o:o + n].zero_()
            self.bufs["v"][o:o + n].zero_()
        hp = N.make_hparams(auto_sync=auto_sync, **hyper)
        descs = [N.novak_tensor_desc(*(self.bufs[r].data_ptr() + self.bufs[r].element_size() * o for r in ("theta", "m", "v", "la")), n)
                 for o, n in zip(self.offsets, self.numels)]
        rc, self.handle = N.novak_create(hp, descs, 0)
        N.check(rc, "novak_create")
        rc, info = N.novak_get_info(self.handle)
        self.h = H.oracle_hyper(hyper, H.NEST_NAMES[info.nesterov_mode], H.LA_NAMES[info.lookahead_mode], info)
        self.auto_sync = auto_sync
        if self.h.lookahead != "none":
            N.check(N.novak_lookahead_init(self.handle, 0), "lookahead_init", self.handle)
        self.state = O.init_state(self.bufs["theta"][self.idx].cpu().numpy(), self.h)
        # a bfloat16 m is a discontinuous decision: such runs are compared after every step from a common state
        self.checked = H.CheckedOracle([self.state], self.h, self.wl.grad_dtype) if H.needs_common_state(self.h) else None
        self.t = 0

    def _sampled(self, role):
        return self.bufs[role][self.idx].float().cpu().numpy()

    def step(self):
        self.t += 1
        t = self.t
        if self.g.dtype == torch.bfloat16:
            tmp = torch.empty(self.flat_len, dtype=torch.float32, device=self.dev)
            tmp.normal_(0.0, self.wl.grad_std, generator=self.gen)
            self.g.copy_(tmp)                      # round-to-nearest-even to bf16
            del tmp
        else:
            self.g.normal_(0.0, self.wl.grad_std, generator=self.gen)
        stream = torch.cuda.current_stream().cuda_stream
        if self.checked is not None:
            self.checked.load([self._sampled("theta")], [self._sampled("m")], [self._sampled("v")])
        N.check(N.novak_step(self.handle, self._grad_arr, N.GRAD_DTYPE[self.wl.grad_dtype], t, stream), f"step {t}", self.handle)
        if (not self.auto_sync) and O.sync_due(t, self.h):
            N.check(N.novak_lookahead_sync(self.handle, stream), f"sync {t}", self.handle)
        g_s = self.g[self.idx].float().cpu().numpy()
        if self.checked is not None:
            self.checked.step([g_s], t, [self._sampled("theta")], [self._sampled("m")], [self._sampled("v")], tag=f"{self.wl.name} ")
            self.state = self.checked.states[0]
            return
        O.step(self.state, g_s, t, self.h)
        if O.sync_due(t, self.h):
            O.lookahead_sync(self.state, self.h)

    def check(self, tag):
        torch.cuda.synchronize()
        if self.checked is not None:
            self.checked.finish(self.t)
        for role, ref in (("theta", self.state.theta), ("m", self.state.m), ("v", self.state.v)):
            got = self._sampled(role)
            H.assert_close(f"{tag} {role}", got, ref)
            H.assert_close_strict(f"{tag} {role}", got, ref)
        if self.h.lookahead == "memory_efficient" and not (self.auto_sync and self.t % self.h.la_k == 0):
            ref = H.blend_buffer(self.state, self.h) if self.state.window else self.state.theta
            H.assert_close(f"{tag} la", self._sampled("la"), ref)
        if self.h.lookahead == "basic":
            H.assert_close(f"{tag} slow", self._sampled("la"), self.state.slow0)
        # whole-buffer properties: nothing outside the tensors was written (every gap of every role), finite, v >= 0
        for r in ("theta", "m", "v", "la"):
            assert bool((self.bufs[r][self.outside] == SENTINEL).all()), f"{tag}: {r} written outside its tensors"
        assert bool(torch.isfinite(self.bufs["theta"]).all())
        assert float(self.bufs["v"].min()) >= 0.0

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            N.novak_destroy(self.handle)
            self.handle = None
        if self.arena is not None:
            torch.cuda.synchronize()
            self.bufs, self.g, self.arena = {}, None, None
            N.check(N.novak_arena_free(0, self.arena_ptr), "novak_arena_free")


def test_c2_resnet50_fast_path_100_steps():
    wl = W.get_workload("c2_resnet50")
    run = FullRun(wl)
    try:
        run.reset(wl.hyper)
        for t in range(1, 101):
            run.step()
            if t in (10, 100):
                run.check(f"c2 t={t}")
        _say("c2 done")
    finally:
        run.close()


def test_c3_vgg16_fast_and_research_modes_100_steps():
    """The stated horizon (100 fp32 steps, 20 lookahead windows) on the 138M-parameter list."""
    wl = W.get_workload("c3_vgg16")
    run = FullRun(wl)
    try:
        for name, hyper, auto in (("fast", wl.hyper, False),
                                  ("fast-auto_sync", wl.hyper, True),
                                  ("research-basic-classical", dict(wl.hyper, mode="research", lookahead="basic", nesterov="classical"), False)):
            run.reset(hyper, auto_sync=auto)
            for t in range(1, 101):
                run.step()
                if t in (4, 10, 11, 50, 100):
                    run.check(f"c3 {name} t={t}")
            _say(f"c3 {name} done")
    finally:
        run.close()


@pytest.mark.parametrize("seed", [100, 2025])
def test_c3_vgg16_other_seeds_of_the_papers_experiments(seed):
    """Section 9.1 runs every experiment under seeds 42, 100 and 2025; the other tests use 42."""
    wl = W.get_workload("c3_vgg16")
    run = FullRun(wl, seed=seed)
    try:
        run.reset(wl.hyper, auto_sync=True)
        for t in range(1, 12):
            run.step()
            if t in (5, 11):
                run.check(f"c3 seed={seed} t={t}")
        _say(f"c3 seed {seed} done")
    finally:
        run.close()


def test_c4_vit_b16_bf16_gradients_100_steps():
    wl = W.get_workload("c4_vit_b16_bf16")
    run = FullRun(wl, arena=True)          # odd tensor sizes (1000, 197 x 768, ...): padding inside the roles
    try:
        run.reset(wl.hyper)
        for t in range(1, 101):
            run.step()
            if t in (7, 100):
                run.check(f"c4 t={t}")
        _say("c4 done")
    finally:
        run.close()


def test_c5_decoder_1p3b_sweep():
    """1.3B parameters (5.26 GB per buffer, offsets beyond 2^31 bytes): k in {5,10} x Nesterov variants."""
    wl = W.get_workload("c5_decoder_1p3b")
    run = FullRun(wl, samples_per_tensor=1024)
    try:
        for k in (5, 10):
            for nest in ("none", "approx", "classical", "true"):
                hyper = dict(wl.hyper, la_k=k, nesterov=nest, mode="research")
                run.reset(hyper)
                for t in range(1, 2 * k + 2):
                    run.step()
                    if t in (k - 1, 2 * k, 2 * k + 1):
                        run.check(f"c5 k={k} {nest} t={t}")
                _say(f"c5 k={k} nesterov={nest} done")
        # the exact configuration bench.py times: fast mode, approximation, k = 5, sync fused into the k-th step,
        # all roles in one allocation placed by novak_plan_arena
        run.close()
        del run
        torch.cuda.empty_cache()
        run = FullRun(wl, samples_per_tensor=1024, arena=True)
        run.reset(wl.hyper, auto_sync=True)
        for t in range(1, 101):
            run.step()
            if t in (4, 5, 6, 10, 11, 50, 100):
                run.check(f"c5 bench-config t={t}")
        _say("c5 bench configuration done (100 steps)")
        # one point of the sweep over the stated horizon as well: k = 10, separate sync kernel
        run.reset(dict(wl.hyper, la_k=10), auto_sync=False)
        for t in range(1, 101):
            run.step()
            if t in (9, 50, 100):
                run.check(f"c5 k=10 t={t}")
        _say("c5 k=10 done (100 steps)")
    finally:
        run.close()


def test_c2_resnet50_every_element_fast_path():
    """The single-pass kernel against the oracle on EVERY element of the ResNet-50 list (25.6M), arena layout."""
    wl = W.get_workload("c2_resnet50")
    run = FullRun(wl, arena=True, dense="all")
    try:
        assert run.idx_host.size == wl.total
        run.reset(wl.hyper, auto_sync=True)
        for t in range(1, 11):
            run.step()
            if t in (4, 5, 10):
                run.check(f"c2 dense t={t}")
            _say(f"c2 dense step {t} done")
    finally:
        run.close()


@pytest.mark.parametrize("name,steps,auto_sync", [("c4_vit_b16_bf16", 6, True), ("c3_vgg16", 6, False)])
def test_every_element_of_the_other_large_lists(name, steps, auto_sync):
    """Every element of the ViT-B/16 list (bf16 gradients: the 64-bit gradient path, odd tensor sizes in a padded
    arena) and of the VGG-16 list (one tensor of 102.8M elements: 6272 chunks; separate sync kernel) across a sync."""
    wl = W.get_workload(name)
    run = FullRun(wl, arena=True, dense="all")
    try:
        assert run.idx_host.size == wl.total
        run.reset(wl.hyper, auto_sync=auto_sync)
        for t in range(1, steps + 1):
            run.step()
            if t in (4, 5, steps):
                run.check(f"{name} dense t={t}")
            _say(f"{name} dense step {t} done")
    finally:
        run.close()


def test_c5_one_whole_large_tensor_every_element():
    """Every element of one 8192 x 2048 tensor (16.7M elements, 1024 chunks) in the middle of the 1.3B list, in the
    configuration bench.py times (arena, sync fused), over 2k+1 steps; the other tensors are sampled."""
    wl = W.get_workload("c5_decoder_1p3b")
    which = next(i for i, s in enumerate(wl.shapes) if s == (8192, 2048) and i > len(wl.shapes) // 2)
    run = FullRun(wl, samples_per_tensor=256, arena=True, dense=(which,))
    try:
        assert run.idx_host.size > 8192 * 2048
        run.reset(wl.hyper, auto_sync=True)
        for t in range(1, 12):
            run.step()
            if t in (4, 5, 6, 11):
                run.check(f"c5 dense tensor {which} t={t}")
            _say(f"c5 dense step {t} done")
    finally:
        run.close()


def test_c5_bf16_first_moment_bench_config():
    """The reduced-precision configuration bench.py can time: 1.3B parameters, m in bfloat16."""
    wl = W.get_workload("c5_decoder_1p3b")
    run = FullRun(wl, samples_per_tensor=1024, arena=True)
    try:
        run.reset(dict(wl.hyper, moment_dtype="bf16_m"), auto_sync=True)
        for t in range(1, 26):
            run.step()            # every step checks every sampled element (common state)
            if t in (4, 5, 6, 10, 11, 25):
                run.check(f"c5 bf16-m t={t}")
        _say("c5 bf16 m done")
    finally:
        run.close()


def test_c4_bf16_gradients_and_bf16_first_moment():
    """Both 2-byte streams at once on the ViT-B/16 list (odd tensor sizes, padded arena), over the
    100-step horizon: with bfloat16 gradients about one rounding in a hundred sits on an exact tie."""
    wl = W.get_workload("c4_vit_b16_bf16")
    run = FullRun(wl, arena=True)
    try:
        run.reset(dict(wl.hyper, moment_dtype="bf16_m"), auto_sync=True)
        for t in range(1, 101):
            run.step()            # every step checks every sampled element (common state)
            if t in (4, 5, 7, 50, 100):
                run.check(f"c4 bf16 g+m t={t}")
        _say("c4 bf16 g+m done")
    finally:
        run.close()


def test_single_tensor_beyond_2_31_elements():
    """Maximum-size edge case: one tensor of 2^31 + 4099 elements (element offsets need 64 bits, the
    element count is odd so the last sub-block has a ragged tail), plus a tiny neighbour."""
    big = (1 << 31) + 4099
    wl = W.Workload("huge_single", ((big,), (7,)), 1e-3, "f32", 6, dict(W.BASE_HYPER))
    run = FullRun(wl, samples_per_tensor=4096)
    try:
        # make sure the far end of the tensor is among the samples
        assert int(run.idx_host.max()) > (1 << 31)
        run.reset(wl.hyper)
        for t in range(1, 7):
            run.step()
            if t in (1, 5, 6):
                run.check(f"huge t={t}")
        _say("huge done")
    finally:
        run.close()
