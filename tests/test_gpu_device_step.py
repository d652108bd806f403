"""Device-step mode: the step count lives in device memory and the scalar prologue runs in a small kernel on the device, so a
captured novak_step advances by itself on every graph replay.  Checked against the oracle like the host-step path,
against the host-step path itself, and - captured into a HIP graph through torch - on every one of many replays with
eager work and synchronisations in between."""
import ctypes as C
import warnings

import numpy as np
import pytest
import torch

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nesterov,lookahead,k,grad_dtype,extra", [
    ("approx", "memory_efficient", 5, "f32", {}),
    ("classical", "basic", 3, "bf16", {}),
    ("none", "none", 5, "f32", {"unrect_fallback": "sgdm"}),
    ("true", "memory_efficient", 1, "f32", {"n_taylor": 4}),
    ("approx", "memory_efficient", 4, "bf16", {"moment_dtype": "bf16_m"}),
    ("approx", "memory_efficient", 5, "f32", {"adaptive_beta": True, "clip_threshold": 0.5, "sparse_threshold": 0.1}),
    ("approx", "memory_efficient", 5, "f32", {"use_gc": True, "clip_threshold": 0.7}),
    # the two-pass step (trust ratio, automatic rate): research mode
    ("approx", "memory_efficient", 5, "f32", {"mode": "research", "layer_adaptation": True, "auto_lr": True}),
    ("classical", "basic", 3, "bf16", {"mode": "research", "layer_adaptation": True, "clip_threshold": 0.6}),
    ("none", "none", 5, "f32", {"mode": "research", "auto_lr": True, "moment_dtype": "bf16_m"}),
    ("approx", "memory_efficient", 1, "f32", {"mode": "research", "layer_adaptation": True, "auto_lr": True, "use_gc": True}),
])
def test_ragged_against_the_oracle(nesterov, lookahead, k, grad_dtype, extra):
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, nesterov=nesterov, lookahead=lookahead, la_k=k, device_step=True, **extra)
    gpu, states, h = H.run_pair(wl.numels, hyper, 2 * k + 13, wl.grad_std, grad_dtype, auto_sync=True, guard=8,
                                rows=wl.rows if extra.get("use_gc") else None)
    try:
        H.compare_states(gpu, states)
        assert gpu.guards_intact()
        assert int(gpu.counter.item()) == 2 * k + 13
    finally:
        gpu.close()


def test_matches_the_host_step_path():
    """Same kernels, constants from a device-side double evaluation instead of the host's: the fp32 constants agree
    (device and host libm may differ in the last bit of a double, which the rounding to fp32 all but always hides)."""
    wl = W.get_workload("ragged")
    a, _, _ = H.run_pair(wl.numels, dict(wl.hyper, device_step=True), 23, wl.grad_std, auto_sync=True)
    b, _, _ = H.run_pair(wl.numels, dict(wl.hyper), 23, wl.grad_std, auto_sync=True)
    try:
        for role in ("theta", "m", "v"):
            for x, y in zip(a.host(role), b.host(role)):
                np.testing.assert_allclose(x, y, rtol=2e-6, atol=1e-9)
        same = sum(int(np.array_equal(x, y)) for x, y in zip(a.host("theta"), b.host("theta")))
        assert same >= len(wl.numels) - 1, "the two prologues should round to the same fp32 constants"
    finally:
        a.close()
        b.close()


def test_resume_from_a_counter_value():
    wl = W.get_workload("ragged")
    numels = wl.numels[:9]
    hyper = dict(wl.hyper, device_step=True)
    full, _, _ = H.run_pair(numels, hyper, 15, wl.grad_std, auto_sync=True)
    part, _, _ = H.run_pair(numels, hyper, 10, wl.grad_std, auto_sync=True)
    descs = [N.novak_tensor_desc(part.theta[i].data_ptr(), part.m[i].data_ptr(), part.v[i].data_ptr(), part.la[i].data_ptr(), n)
             for i, n in enumerate(numels)]
    part.close()
    rc, handle = N.novak_create(N.make_hparams(auto_sync=True, **hyper), descs, 0)
    N.check(rc, "create")
    part.handle = handle
    try:
        g = part.upload_grads(W.host_grads(numels, 11, wl.grad_std))
        assert part.step(11, g) == N.NOVAK_ERR_STATE                          # no counter yet
        assert N.novak_set_step_counter(handle, part.counter.data_ptr() + 4) == N.NOVAK_ERR_MISALIGNED
        N.check(N.novak_set_step_counter(handle, part.counter.data_ptr()), "counter", handle)     # still holds 10
        for t in range(11, 16):
            N.check(part.step(t, part.upload_grads(W.host_grads(numels, t, wl.grad_std))), "step", handle)
        for role in ("theta", "m", "v"):
            for x, y in zip(full.host(role), part.host(role)):
                assert np.array_equal(x, y)
    finally:
        full.close()
        part.close()


def test_rules_of_the_mode():
    d = N.novak_tensor_desc(4096, 8192, 12288, 16384, 64)
    assert N.novak_create(N.make_hparams(device_step=True, auto_sync=False), [d])[0] == N.NOVAK_ERR_INVALID_ARG
    assert "auto_sync" in N.novak_last_error()
    t = torch.zeros(4, 64, device="cuda:0")
    real = N.novak_tensor_desc(t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), t[3].data_ptr(), 64)
    rc, h = N.novak_create(N.make_hparams(device_step=True, auto_sync=True), [real], 0)
    N.check(rc, "create")
    try:
        g = (C.c_void_p * 1)(t[0].data_ptr())
        assert N.novak_step(h, g, N.NOVAK_GRAD_F32, 1, 0) == N.NOVAK_ERR_BAD_STEP          # step must be 0 in this mode
        assert N.novak_step(h, g, N.NOVAK_GRAD_F32, 0, 0) == N.NOVAK_ERR_STATE             # counter missing
        assert N.novak_lookahead_sync(h, 0) == N.NOVAK_ERR_STATE
        assert N.novak_step_static(N.make_hparams(device_step=True, auto_sync=True), [real], g, 0, 1) == N.NOVAK_ERR_INVALID_ARG
    finally:
        N.novak_destroy(h)
    rc, h = N.novak_create(N.make_hparams(auto_sync=True), [real], 0)
    assert N.novak_set_step_counter(h, t.data_ptr()) == N.NOVAK_ERR_STATE                 # host-step handle
    N.novak_destroy(h)


def test_a_list_without_elements_still_counts_its_steps():
    counter = torch.full((1,), 7, dtype=torch.int64, device="cuda:0")
    for descs, grads in (([], []), ([N.novak_tensor_desc(0, 0, 0, 0, 0)], (C.c_void_p * 1)(0))):
        rc, h = N.novak_create(N.make_hparams(device_step=True, auto_sync=True), descs, 0)
        N.check(rc, "create")
        try:
            N.check(N.novak_set_step_counter(h, counter.data_ptr()), "counter", h)
            before = int(counter.item())
            for _ in range(3):
                N.check(N.novak_step(h, grads, N.NOVAK_GRAD_F32, 0, torch.cuda.current_stream().cuda_stream), "step", h)
            assert int(counter.item()) == before + 3
        finally:
            N.novak_destroy(h)


@pytest.mark.parametrize("lookahead,k,extra", [("memory_efficient", 5, {}), ("none", 5, {}), ("basic", 2, {}),
                                               ("memory_efficient", 4, {"mode": "research", "layer_adaptation": True, "auto_lr": True})])
def test_captured_step_advances_on_every_replay(lookahead, k, extra):
    """One novak_step captured into a HIP graph (through torch's stream capture) and replayed 17 times; before every
    replay new gradients are written into the captured buffers by ordinary eager work, after it the program
    synchronises and compares the whole state with an eager host-step twin that took the same steps."""
    wl = W.get_workload("ragged")
    numels = wl.numels
    hyper = dict(wl.hyper, lookahead=lookahead, la_k=k, clip_threshold=0.8, **extra)
    theta0 = W.host_params(numels, 7)
    cap = H.GpuNovak(numels, dict(hyper, device_step=True), "f32", theta0, auto_sync=True)
    twin = H.GpuNovak(numels, hyper, "f32", theta0, auto_sync=True)
    try:
        static_g = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in numels]

        def load(t):
            gh = W.host_grads(numels, t, wl.grad_std, 7)
            for dst, src in zip(static_g, gh):
                dst.copy_(torch.from_numpy(src))
            return gh

        def check(t):
            torch.cuda.synchronize()
            for role in ("theta", "m", "v"):
                for i, (x, y) in enumerate(zip(cap.host(role), twin.host(role))):
                    np.testing.assert_allclose(x, y, rtol=2e-6, atol=1e-9, err_msg=f"{role}[{i}] after step {t}")

        # step 1 eagerly: uploads the gradient-pointer list, which a capture cannot
        load(1)
        N.check(cap.step(1, static_g), "eager step 1", cap.handle)
        N.check(twin.step(1, static_g), "twin step 1", twin.handle)
        check(1)
        load(2)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            N.check(N.novak_step(cap.handle, cap._grad_arr, N.NOVAK_GRAD_F32, 0, torch.cuda.current_stream().cuda_stream), "captured step", cap.handle)
        # the capture itself executed nothing: the counter still says 1
        assert int(cap.counter.item()) == 1
        for t in range(2, 19):
            load(t)                                        # eager work between replays
            graph.replay()
            N.check(twin.step(t, static_g), f"twin step {t}", twin.handle)
            check(t)
            assert int(cap.counter.item()) == t
        del graph
    finally:
        cap.close()
        twin.close()


def test_captures_are_self_contained():
    """Under capture one prologue writes the records of 64 steps ahead and the captured steps take them in turn.  So:
    a capture that was never replayed must leave nothing behind for the eager steps that follow; two graphs captured
    back to back must not share records; a graph of more than 64 steps writes records twice; and graphs, replayed in
    any order between eager steps, must each continue from the device's counter.  An eager host-step twin takes the
    same steps on the same gradients."""
    wl = W.get_workload("ragged")
    numels = wl.numels[:8]
    hyper = dict(wl.hyper, lookahead="memory_efficient", la_k=3)
    theta0 = W.host_params(numels, 11)
    cap = H.GpuNovak(numels, dict(hyper, device_step=True), "f32", theta0, auto_sync=True)
    twin = H.GpuNovak(numels, hyper, "f32", theta0, auto_sync=True)
    try:
        static_g = cap.upload_grads(W.host_grads(numels, 1, wl.grad_std, 11))
        state = {"t": 0}

        def twin_steps(n):
            for _ in range(n):
                state["t"] += 1
                N.check(twin.step(state["t"], static_g), f"twin step {state['t']}", twin.handle)

        def eager():
            N.check(cap.step(state["t"] + 1, static_g), "eager step", cap.handle)
            twin_steps(1)

        def capture(n):
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(n):
                    N.check(N.novak_step(cap.handle, cap._grad_arr, N.NOVAK_GRAD_F32, 0, torch.cuda.current_stream().cuda_stream),
                            "captured step", cap.handle)
            return g

        def check(tag):
            torch.cuda.synchronize()
            assert int(cap.counter.item()) == state["t"], tag
            for role in ("theta", "m", "v"):
                for i, (x, y) in enumerate(zip(cap.host(role), twin.host(role))):
                    np.testing.assert_allclose(x, y, rtol=2e-6, atol=1e-9, err_msg=f"{tag}: {role}[{i}]")

        # a capture may not upload a gradient-pointer list: refused with a reason, and the capture goes on
        other_g = [g.clone() for g in static_g]
        other = (C.c_void_p * len(numels))(*[g.data_ptr() for g in other_g])
        torch.cuda.synchronize()
        probe = torch.cuda.CUDAGraph()
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")           # torch remarks that the captured graph is empty: that is the point
            with torch.cuda.graph(probe):
                rc = N.novak_step(cap.handle, other, N.NOVAK_GRAD_F32, 0, torch.cuda.current_stream().cuda_stream)
        assert rc == N.NOVAK_ERR_STATE and "captured" in N.novak_last_error(cap.handle)
        del probe
        eager()                                   # t = 1: uploads the gradient-pointer list
        graph_a = capture(3)
        graph_b = capture(70)                     # right behind the first capture; crosses the 64-record boundary
        check("captures execute nothing")
        eager()                                   # t = 2, although 73 steps were captured in between
        check("eager step after two captures that never ran")
        graph_a.replay(); twin_steps(3); check("first replay of the short graph")
        eager(); check("eager step after a replay")
        graph_b.replay(); twin_steps(70); check("the long graph")
        graph_a.replay(); twin_steps(3); check("the short graph after the long one")
        graph_b.replay(); twin_steps(70)
        eager(); check("at the end")
        assert state["t"] == 150
        del graph_a, graph_b
    finally:
        cap.close()
        twin.close()
