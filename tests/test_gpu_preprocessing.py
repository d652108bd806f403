"""GPU parity of gradient clipping (global norm, sections 5.8 / 7.3) and the sparse threshold (Eq. 27)."""
import numpy as np
import pytest

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("clip,tau", [(1.0, 0.0), (0.0, 0.3), (1.0, 0.3), (1e6, 0.0)])
@pytest.mark.parametrize("nesterov,lookahead,grad_dtype,two_pass,mode", [
    ("approx", "memory_efficient", "f32", False, "fast"), ("approx", "memory_efficient", "bf16", False, "research"),
    ("classical", "basic", "f32", True, "research"), ("none", "none", "bf16", True, "research")])
def test_ragged_clip_and_sparse(clip, tau, nesterov, lookahead, grad_dtype, two_pass, mode):
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, mode=mode, nesterov=nesterov, lookahead=lookahead, clip_threshold=clip, sparse_threshold=tau,
                 layer_adaptation=two_pass, auto_lr=two_pass)
    print(f"prep {clip} {tau} {nesterov} {lookahead} {grad_dtype} {two_pass} {mode}", flush=True)
    gpu, states, h = H.run_pair(wl.numels, hyper, wl.steps, wl.grad_std, grad_dtype, auto_sync=True, chunk_elems=4096, guard=16)
    try:
        H.compare_states(gpu, states)
        assert gpu.guards_intact()
    finally:
        gpu.close()
    if clip == 1.0:
        # the clip really bites on this workload: global norm of N(0, 1e-2) over 5.2e5 elements is ~7
        g = W.host_grads(wl.numels, 1, wl.grad_std, bf16=(grad_dtype == "bf16"))
        assert O.clip_scale(g, O.Hyper(clip_threshold=1.0)) < 0.2


def test_clip_with_misaligned_buffers_and_coupled_decay():
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, clip_threshold=0.5, sparse_threshold=0.1, decoupled_decay=False, weight_decay=0.05, unrect_fallback="sgdm")
    gpu, states, _ = H.run_pair(wl.numels, hyper, 7, wl.grad_std, misalign=3, grad_misalign=1, guard=8)
    try:
        H.compare_states(gpu, states)
        assert gpu.guards_intact()
    finally:
        gpu.close()


def test_sparse_mask_zeroes_small_directions_exactly():
    """Elements whose |u| <= tau do not move at all (decay off): bit-equal to their initial value."""
    n = [4096]
    theta0 = W.host_params(n)
    g = W.host_grads(n, 1, 1e-2)[0].copy()
    g[::2] = 1e-12                                    # u = g/(|g|+1e-8) ~ 1e-4 for these
    hyper = dict(W.BASE_HYPER, weight_decay=0.0, nesterov="none", lookahead="none", sparse_threshold=0.5)
    gpu = H.GpuNovak(n, hyper, "f32", theta0)
    try:
        N.check(gpu.step(1, gpu.upload_grads([g])), "step", gpu.handle)
        th = gpu.host("theta")[0]
        assert np.array_equal(th[::2], theta0[0][::2])
        assert np.all(th[1::2] != theta0[0][1::2])
    finally:
        gpu.close()


GC_SHAPES = [(64, 3, 7, 7), (64,), (256, 64, 1, 1), (5, 1021), (1000, 2048), (1000,), (3, 5, 7), (4099, 1), (1, 4097), (2, 65536 + 3)]


@pytest.mark.parametrize("grad_dtype,two_pass,clip,misalign", [("f32", False, 0.0, 0), ("bf16", False, 1.0, 0), ("f32", True, 1.0, 0),
                                                               ("f32", False, 0.0, 1), ("bf16", True, 0.0, 3)])
def test_gradient_centralization(grad_dtype, two_pass, clip, misalign):
    """Eq. 26 on conv / linear shaped tensors: rows of 147, 64, 1021, 2048 elements, one-element rows
    (the centralized gradient is zero), one single long row, and vectors that are left alone."""
    numels = [int(np.prod(s)) for s in GC_SHAPES]
    rows = [s[0] if len(s) > 1 else 0 for s in GC_SHAPES]
    hyper = dict(W.BASE_HYPER, mode="research", use_gc=True, clip_threshold=clip, layer_adaptation=two_pass, auto_lr=two_pass)
    print(f"gc {grad_dtype} {two_pass} {clip} {misalign}", flush=True)
    gpu, states, h = H.run_pair(numels, hyper, 7, 1e-2, grad_dtype, auto_sync=True, rows=rows, guard=8,
                                misalign=misalign, grad_misalign=misalign)
    try:
        assert gpu.info.use_gc == 1 and gpu.info.n_centralized == sum(1 for r in rows if r >= 1)
        H.compare_states(gpu, states)
        assert gpu.guards_intact()
        # rows of one element: the centralized gradient is exactly zero, so m stays zero
        assert not gpu.host("m")[7].any()
    finally:
        gpu.close()


def test_centralization_changes_results_and_fast_mode_switches_it_off():
    numels = [int(np.prod(s)) for s in GC_SHAPES[:4]]
    rows = [s[0] if len(s) > 1 else 0 for s in GC_SHAPES[:4]]
    on, st_on, _ = H.run_pair(numels, dict(W.BASE_HYPER, mode="research", use_gc=True), 3, 1e-2, rows=rows)
    off, st_off, _ = H.run_pair(numels, dict(W.BASE_HYPER, mode="fast", use_gc=True), 3, 1e-2, rows=rows)
    try:
        assert off.info.use_gc == 0 and off.info.warnings & N.NOVAK_WARN_GC_DISABLED
        H.compare_states(on, st_on)
        H.compare_states(off, st_off)
        assert np.max(np.abs(on.host("theta")[0] - off.host("theta")[0])) > 1e-6
    finally:
        on.close()
        off.close()


def test_rows_must_divide_numel():
    hp = N.make_hparams(mode="research", use_gc=True, lookahead="none")
    assert N.novak_create(hp, [N.novak_tensor_desc(256, 512, 768, None, 10, 3)])[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_create(hp, [N.novak_tensor_desc(256, 512, 768, None, 10, -1)])[0] == N.NOVAK_ERR_INVALID_ARG


def test_row_means_do_not_depend_on_chunking_or_prepass_residency():
    """The pre-pass sums rows in spans of 4096 elements counted from the tensor's start, whatever the chunk
    size (1, 4 or 16 spans per chunk-table entry: the last exercises the pipelined two-buffer loop) and
    whatever its residency: centralized results are bit-identical.  With clipping on, only the grouping of
    the norm's partial sums changes, so those runs are compared with the oracle instead."""
    shapes = GC_SHAPES + [(96, 1024), (40, 4096 + 256), (3, 70000)]
    numels = [int(np.prod(s)) for s in shapes]
    rows = [s[0] if len(s) > 1 else 0 for s in shapes]
    hyper = dict(W.BASE_HYPER, mode="research", use_gc=True)
    outs = []
    for chunk, waves in ((4096, 0), (16384, 0), (65536, 0), (65536, 3), (16384, 32)):
        gpu, states, _ = H.run_pair(numels, hyper, 6, 1e-2, auto_sync=True, rows=rows, chunk_elems=chunk)
        N.check(N.novak_set_tuning(gpu.handle, N.NOVAK_TUNE_PREPASS_WAVES_PER_CU, waves), "set_tuning", gpu.handle)
        gh = W.host_grads(numels, 7, 1e-2)
        N.check(gpu.step(7, gpu.upload_grads(gh)), "step 7", gpu.handle)
        outs.append([gpu.host(r) for r in ("theta", "m", "v")])
        gpu.close()
    for other in outs[1:]:
        for role_a, role_b in zip(outs[0], other):
            for x, y in zip(role_a, role_b):
                assert np.array_equal(x, y)
    for chunk in (4096, 65536):
        gpu, states, _ = H.run_pair(numels, dict(hyper, clip_threshold=0.7), 6, 1e-2, auto_sync=True, rows=rows, chunk_elems=chunk, guard=8)
        try:
            H.compare_states(gpu, states)
            assert gpu.guards_intact()
        finally:
            gpu.close()
