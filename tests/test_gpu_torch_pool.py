"""The allocator hooks for PyTorch (novak_torch_malloc / novak_torch_free through torch.cuda.MemPool): tensors a
caller creates inside the pool live in memory the library allocated (physically contiguous when the driver can),
behave like any other torch tensors, and the update step on them matches the oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N
from tests import harness as H

pytestmark = pytest.mark.gpu


def test_step_on_tensors_from_the_pool_matches_the_oracle():
    wl = W.get_workload("ragged")
    numels = wl.numels + [3 << 20]                       # one tensor large enough for a segment of its own
    theta0 = W.host_params(numels, 2025)
    live0, _ = N.novak_torch_alloc_stats()
    pool = N.torch_mem_pool()
    with torch.cuda.use_mem_pool(pool):
        theta = [torch.from_numpy(t).to("cuda:0") for t in theta0]
        m = [torch.zeros_like(t) for t in theta]
        v = [torch.zeros_like(t) for t in theta]
        la = [t.clone() for t in theta]
        g = [torch.empty_like(t) for t in theta]
    live, contiguous = N.novak_torch_alloc_stats()
    assert live > live0, "torch did not take the pool's segments from the library"
    print(f"pool: {live - live0} segments from novak_torch_malloc, {contiguous} physically contiguous", flush=True)
    # ordinary torch semantics on that memory
    assert float(m[-1].sum()) == 0.0 and torch.equal(la[0], theta[0])
    hyper = dict(wl.hyper)
    hp = N.make_hparams(auto_sync=True, **hyper)
    descs = [N.tensor_desc(*x) for x in zip(theta, m, v, la)]
    rc, handle = N.novak_create(hp, descs, 0)
    N.check(rc, "novak_create")
    h = H.oracle_hyper(hyper)
    states = [O.init_state(t, h) for t in theta0]
    try:
        stream = torch.cuda.current_stream().cuda_stream
        for t in range(1, 8):
            gh = W.host_grads(numels, t, wl.grad_std, 2025)
            for dst, src in zip(g, gh):
                dst.copy_(torch.from_numpy(src))
            N.check(N.novak_step(handle, [x.data_ptr() for x in g], N.NOVAK_GRAD_F32, t, stream), f"step {t}", handle)
            O.step_all(states, gh, t, h)
            if O.sync_due(t, h):
                for st in states:
                    O.lookahead_sync(st, h)
        torch.cuda.synchronize()
        for i, st in enumerate(states):
            for role, got in (("theta", theta[i]), ("m", m[i]), ("v", v[i])):
                H.assert_close(f"{role}[{i}]", got.cpu().numpy(), getattr(st, role))
    finally:
        torch.cuda.synchronize()
        N.novak_destroy(handle)
    # memory goes back through novak_torch_free once the tensors and the pool are gone
    del theta, m, v, la, g, descs
    del pool
    torch.cuda.empty_cache()
    assert N.novak_torch_alloc_stats()[0] <= live


def test_hooks_directly():
    """The two functions as torch calls them: sizes below and above the 1 MiB mark, the skew of large addresses, frees."""
    lib = N.load_library()
    live0, _ = N.novak_torch_alloc_stats()
    small = lib.novak_torch_malloc(4096, 0, None)
    a = lib.novak_torch_malloc(8 << 20, 0, None)
    b = lib.novak_torch_malloc(8 << 20, 0, None)
    assert small and a and b
    assert (b - a) % N.NOVAK_ARENA_ROLE_PERIOD in (N.NOVAK_ARENA_ROLE_SKEW, N.NOVAK_ARENA_ROLE_PERIOD - 3 * N.NOVAK_ARENA_ROLE_SKEW) or \
        ((b % N.NOVAK_ARENA_ROLE_PERIOD) - (a % N.NOVAK_ARENA_ROLE_PERIOD)) % N.NOVAK_ARENA_ROLE_PERIOD == N.NOVAK_ARENA_ROLE_SKEW
    assert N.novak_torch_alloc_stats()[0] == live0 + 3
    t = N.arena_as_tensor(a, 8 << 20, 0)
    t.fill_(7)
    assert int(t.sum()) == 7 * (8 << 20)
    del t
    torch.cuda.synchronize()
    for p, n in ((small, 4096), (a, 8 << 20), (b, 8 << 20)):
        lib.novak_torch_free(p, n, 0, None)
    lib.novak_torch_free(12345678, 16, 0, None)            # an address that is not ours is left alone
    assert N.novak_torch_alloc_stats()[0] == live0
    assert lib.novak_torch_malloc(-1, 0, None) is None and lib.novak_torch_malloc(16, -1, None) is None
