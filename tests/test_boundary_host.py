"""Host-side logic of the C ABI, exercised without a GPU: the library loads and exports every
declared symbol; validation rules and fast-path downgrades (sections 5.8, 7.3); the scalar prologue
against the oracle; chunk-table coverage; algorithmic byte accounting against the paper's figures."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "novak.h")).read()
    declared = set(re.findall(r"\b(novak_[a-z_]+)\s*\(", header))
    assert declared == set(N.EXPORTS)
    lib = N.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_sizes_match_header_layout():
    assert C.sizeof(N.novak_hparams) == 8 + 7 * 8 + 10 * 4 + 7 * 8 + 2 * 4 + 3 * 8 + 2 * 4
    assert C.sizeof(N.novak_tensor_desc) == 48
    assert C.sizeof(N.novak_chunk) == 16
    hp = N.make_hparams()
    hp.struct_size = 12
    assert N.novak_validate_hparams(hp)[0] == N.NOVAK_ERR_INVALID_ARG


GOOD = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2, beta_n=0.9, la_alpha=0.5, la_k=5)


@pytest.mark.parametrize("field,value", [
    ("lr", 0.0), ("lr", -1e-3), ("lr", float("nan")), ("lr", float("inf")),
    ("beta1", 1.0), ("beta1", -0.1), ("beta2", 1.0), ("beta2", -1e-9),
    ("weight_decay", -1e-9), ("beta_n", 1.0), ("beta_n", -0.5),
    ("eps", 0.0), ("eps", -1e-8), ("la_k", 0), ("la_k", -3),
    ("la_alpha", 0.0), ("la_alpha", 1.0000001), ("la_alpha", -0.5),
    ("beta2", 1.0 - 1e-9),                      # rho_inf ill-defined when rectified
    ("clip_threshold", -1.0), ("sparse_threshold", -1e-9), ("clip_threshold", float("nan")),
])
def test_validation_rejects(field, value):
    kw = dict(GOOD)
    kw[field] = value
    rc, _, _ = N.novak_validate_hparams(N.make_hparams(**kw))
    assert rc == N.NOVAK_ERR_INVALID_ARG


def test_validation_accepts_edges():
    for kw in (dict(beta1=0.0), dict(beta2=0.0, rectified=False), dict(weight_decay=0.0), dict(beta_n=0.0),
               dict(la_alpha=1.0), dict(la_k=1), dict(beta2=1.0 - 1e-9, rectified=False),
               dict(la_alpha=5.0, lookahead="none")):
        rc, _, _ = N.novak_validate_hparams(N.make_hparams(**dict(GOOD, **kw)))
        assert rc == N.NOVAK_OK, kw
    for bad in (dict(nesterov=4), dict(lookahead=3), dict(unrect_fallback=2), dict(mode=2), dict(nesterov=-1)):
        assert N.novak_validate_hparams(N.make_hparams(**dict(GOOD, **bad)))[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.load_library().novak_validate_hparams(None, None, None) == N.NOVAK_ERR_NULL_POINTER


def test_scaling_features_validation_and_fast_mode_switch_off():
    ok = dict(GOOD, mode="research", layer_adaptation=True, auto_lr=True)
    rc, eff, warn = N.novak_validate_hparams(N.make_hparams(**ok))
    assert (rc, eff.layer_adaptation, eff.auto_lr, warn) == (0, 1, 1, 0)
    for bad in (dict(trust_clip=(0.0, 10.0)), dict(trust_clip=(2.0, 1.0)), dict(auto_clip=(-1.0, 2.0)), dict(auto_clip=(3.0, 2.0)),
                dict(auto_lr_gamma=0.0), dict(auto_lr_gamma=1.5), dict(auto_lr_gamma=float("nan"))):
        assert N.novak_validate_hparams(N.make_hparams(**dict(ok, **bad)))[0] == N.NOVAK_ERR_INVALID_ARG, bad
    # the ranges are not checked when the feature is off
    assert N.novak_validate_hparams(N.make_hparams(**dict(GOOD, trust_clip=(0.0, 0.0), auto_lr_gamma=0.0)))[0] == N.NOVAK_OK
    rc, eff, warn = N.novak_validate_hparams(N.make_hparams(**dict(ok, mode="fast")))
    assert (rc, eff.layer_adaptation, eff.auto_lr) == (0, 0, 0)
    assert warn == N.NOVAK_WARN_LAYER_ADAPTATION_DISABLED | N.NOVAK_WARN_AUTO_LR_DISABLED
    assert N.novak_bytes_per_param_scaled_step(0, N.NOVAK_GRAD_F32, 5, 1, 0) == 40
    assert N.novak_bytes_per_param_scaled_step(N.NOVAK_LOOKAHEAD_MEMORY_EFFICIENT, N.NOVAK_GRAD_BF16, 5, 2, 0) == 46


def test_schedules_in_the_prologue_match_the_oracle():
    kw = dict(GOOD, adaptive_beta=True, beta_tau1=300.0, beta_tau2=700.0, nesterov="true", mode="research", n_taylor=150)
    hp = N.make_hparams(**kw)
    h = O.Hyper(**{k: v for k, v in kw.items() if k != "mode"})
    for t in (1, 2, 50, 150, 151, 1000, 10 ** 5):
        rc, s = N.novak_compute_step_scalars(hp, t)
        b1, b2 = O.scheduled_betas(h, t)
        assert rc == 0 and s.beta1_t == pytest.approx(b1, rel=1e-15) and s.beta2_t == pytest.approx(b2, rel=1e-15)
        assert {1: "approx", 3: "true"}[s.nesterov_mode] == O.effective_nesterov(h, t)
    assert N.novak_validate_hparams(N.make_hparams(**dict(kw, beta_tau1=0.0)))[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_validate_hparams(N.make_hparams(**dict(kw, n_taylor=-1)))[0] == N.NOVAK_ERR_INVALID_ARG


def test_fast_path_downgrades_warn_and_research_mode_does_not():
    rc, eff, warn = N.novak_validate_hparams(N.make_hparams(mode="fast", nesterov="true", lookahead="basic"))
    assert rc == N.NOVAK_OK
    assert eff.nesterov_mode == N.NOVAK_NESTEROV_APPROX and eff.lookahead_mode == N.NOVAK_LOOKAHEAD_MEMORY_EFFICIENT
    assert warn == N.NOVAK_WARN_TRUE_NESTEROV_DOWNGRADED | N.NOVAK_WARN_LOOKAHEAD_DOWNGRADED
    rc, eff, warn = N.novak_validate_hparams(N.make_hparams(mode="research", nesterov="true", lookahead="basic"))
    assert (rc, eff.nesterov_mode, eff.lookahead_mode, warn) == (0, N.NOVAK_NESTEROV_TRUE, N.NOVAK_LOOKAHEAD_BASIC, 0)
    rc, eff, warn = N.novak_validate_hparams(N.make_hparams(mode="fast", nesterov="classical", lookahead="memory_efficient"))
    assert (eff.nesterov_mode, warn) == (N.NOVAK_NESTEROV_CLASSICAL, 0)


@pytest.mark.parametrize("beta2", [0.999, 0.99, 0.95])
@pytest.mark.parametrize("rectified,fallback", [(True, "adam_denom"), (True, "sgdm"), (False, "adam_denom")])
def test_prologue_matches_oracle_scalars(beta2, rectified, fallback):
    hp = N.make_hparams(**dict(GOOD, beta2=beta2, rectified=rectified, unrect_fallback=fallback))
    h = O.Hyper(**dict(GOOD, beta2=beta2, rectified=rectified, unrect_fallback=fallback))
    for t in list(range(1, 30)) + [100, 999, 1000, 1001, 12345, 10 ** 6]:
        rc, s = N.novak_compute_step_scalars(hp, t)
        assert rc == N.NOVAK_OK
        o = O.step_scalars(h, t)
        for name in ("bc1", "bc2", "rho_inf", "rho_t", "r_t", "step_size", "decay"):
            assert getattr(s, name) == pytest.approx(getattr(o, name), rel=4e-16, abs=0), (name, t)
        assert (s.beta1_t, s.beta2_t) == (0.9, beta2)
        assert bool(s.rectified_now) == o.rectified_now and bool(s.denom_on) == o.denom_on
    assert N.novak_compute_step_scalars(hp, 0)[0] == N.NOVAK_ERR_BAD_STEP


@pytest.mark.parametrize("name", W.WORKLOAD_NAMES + ("ragged",))
@pytest.mark.parametrize("chunk", [4096, 16384, 65536])
def test_chunk_table_covers_every_element_exactly_once(name, chunk):
    numels = W.get_workload(name).numels
    rc, table = N.novak_plan_chunks(numels, chunk)
    assert rc == N.NOVAK_OK
    covered = [0] * len(numels)
    prev = (-1, -1)
    for tensor, off, ln in table:
        assert 0 < ln <= chunk and off % chunk == 0
        assert (tensor, off) > prev            # tensor order, ascending offsets
        assert off == covered[tensor]          # contiguous, no gap, no overlap
        covered[tensor] += ln
        prev = (tensor, off)
    assert covered == list(numels)
    assert len(table) == sum(-(-n // chunk) for n in numels)


def test_chunk_planner_edge_cases():
    assert N.novak_plan_chunks([], 4096) == (N.NOVAK_OK, [])
    assert N.novak_plan_chunks([0, 0], 4096) == (N.NOVAK_OK, [])
    assert N.novak_plan_chunks([1], 4096) == (N.NOVAK_OK, [(0, 0, 1)])
    assert N.novak_plan_chunks([4096, 4097], 4096)[1] == [(0, 0, 4096), (1, 0, 4096), (1, 4096, 1)]
    assert N.novak_plan_chunks([5], 5000)[0] == N.NOVAK_ERR_INVALID_ARG        # not a power of two
    assert N.novak_plan_chunks([5], 12288)[0] == N.NOVAK_ERR_INVALID_ARG       # multiple of 4096, not a power of two
    assert N.novak_plan_chunks([5], 2048)[0] == N.NOVAK_ERR_INVALID_ARG        # below the minimum
    assert N.novak_plan_chunks([5], 0)[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_plan_chunks([-1], 4096)[0] == N.NOVAK_ERR_INVALID_ARG
    # 64-bit offsets: a 3e9-element tensor
    rc, table = N.novak_plan_chunks([3_000_000_000], 1 << 24)
    assert rc == N.NOVAK_OK and table[-1][1] + table[-1][2] == 3_000_000_000 and table[-1][1] > 2 ** 31


def test_algorithmic_bytes_match_the_papers_traffic_arithmetic():
    gold = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_traffic_section_5_5.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            gold[k] = float(v)
    b = N.novak_bytes_per_param_step(N.NOVAK_LOOKAHEAD_NONE, N.NOVAK_GRAD_F32, 5, 1, 0)
    assert b == (gold["streams_read"] + gold["streams_written"]) * gold["bytes_per_element"] == 28
    assert b * gold["params"] == gold["fused_total_bytes"]
    assert gold["read_bytes"] + gold["written_bytes"] == gold["fused_total_bytes"]
    # other variants
    ME, BA, F32, BF = N.NOVAK_LOOKAHEAD_MEMORY_EFFICIENT, N.NOVAK_LOOKAHEAD_BASIC, N.NOVAK_GRAD_F32, N.NOVAK_GRAD_BF16
    assert N.novak_bytes_per_param_step(0, BF, 5, 1, 0) == 26
    assert [N.novak_bytes_per_param_step(ME, F32, 5, p, 0) for p in range(1, 6)] == [32, 36, 36, 36, 36]
    assert [N.novak_bytes_per_param_step(ME, F32, 5, p, 1) for p in range(1, 6)] == [32, 36, 36, 36, 32]
    assert [N.novak_bytes_per_param_step(BA, F32, 5, p, 1) for p in range(1, 6)] == [28, 28, 28, 28, 36]
    assert N.novak_bytes_per_param_step(BA, F32, 5, 5, 0) == 28
    assert N.novak_bytes_per_param_sync(ME) == 8 and N.novak_bytes_per_param_sync(BA) == 16
    assert N.novak_bytes_per_param_sync(0) == 0


def test_create_rejects_bad_arguments_before_touching_the_gpu():
    hp = N.make_hparams(**GOOD)
    d = N.novak_tensor_desc(256, 512, 768, 1024, 8)
    lib = N.load_library()
    h = C.c_void_p()
    assert lib.novak_create(None, C.byref(hp), None, 0, 0) == N.NOVAK_ERR_NULL_POINTER
    assert lib.novak_create(C.byref(h), None, None, 0, 0) == N.NOVAK_ERR_NULL_POINTER
    assert lib.novak_create(C.byref(h), C.byref(hp), None, 2, 0) == N.NOVAK_ERR_NULL_POINTER
    assert lib.novak_create(C.byref(h), C.byref(hp), None, -1, 0) == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_create(N.make_hparams(**dict(GOOD, lr=-1.0)), [d])[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_create(hp, [N.novak_tensor_desc(256, 512, 768, 1024, -8)])[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_create(hp, [N.novak_tensor_desc(0, 512, 768, 1024, 8)])[0] == N.NOVAK_ERR_NULL_POINTER
    assert N.novak_create(hp, [N.novak_tensor_desc(256, 512, 768, 0, 8)])[0] == N.NOVAK_ERR_NULL_POINTER   # lookahead on
    assert N.novak_create(hp, [N.novak_tensor_desc(258, 512, 768, 1024, 8)])[0] == N.NOVAK_ERR_MISALIGNED
    assert "aligned" in N.novak_last_error(None)
    assert N.novak_create(hp, [d], -1)[0] == N.NOVAK_ERR_INVALID_ARG
    # a list that one kernel launch cannot cover (a launch holds < 2^32 threads = 2^26 waves of 256 elements
    # = 2^34 elements) is refused here, with a reason, and not later by the first step; create dereferences
    # nothing, so made-up addresses do
    assert N.novak_create(hp, [N.novak_tensor_desc(1 << 40, 1 << 41, 1 << 42, 1 << 43, 1 << 35)])[0] == N.NOVAK_ERR_INVALID_ARG
    assert "2^32" in N.novak_last_error(None)
    assert N.novak_create(hp, [N.novak_tensor_desc(1 << 40, 1 << 41, 1 << 42, 1 << 43, 1 << 33)] * 2)[0] == N.NOVAK_ERR_INVALID_ARG
    assert "2^32" in N.novak_last_error(None)
    # the allocation-free step makes the same checks before it touches the device
    assert N.novak_step_static(N.make_hparams(**dict(GOOD, lr=-1.0)), [d], [256], 0, 1) == N.NOVAK_ERR_INVALID_ARG
    fused = N.make_hparams(auto_sync=True, **GOOD)
    assert N.novak_step_static(hp, [d], [256], 0, 1) == N.NOVAK_ERR_INVALID_ARG and "auto_sync" in N.novak_last_error(None)
    assert N.novak_step_static(fused, [N.novak_tensor_desc(258, 512, 768, 1024, 8)], [256], 0, 1) == N.NOVAK_ERR_MISALIGNED
    assert N.novak_step_static(fused, [d], [258], 0, 1) == N.NOVAK_ERR_MISALIGNED
    # NULL handle arguments
    assert N.novak_destroy(None) == N.NOVAK_OK
    assert N.novak_step(None, [], 0, 1, 0) == N.NOVAK_ERR_NULL_POINTER
    assert N.novak_lookahead_sync(None, 0) == N.NOVAK_ERR_NULL_POINTER
    assert N.novak_lookahead_init(None, 0) == N.NOVAK_ERR_NULL_POINTER
    assert N.novak_status_string(N.NOVAK_ERR_STATE) != N.novak_status_string(12345)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No fallback path: without the built shared library the binding raises instead of computing elsewhere."""
    monkeypatch.setattr(N, "_lib", None)
    monkeypatch.setattr(N, "LIB_PATH", str(tmp_path / "libnovak.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        N.load_library()
    with pytest.raises(RuntimeError):
        N.novak_validate_hparams(N.make_hparams())


def test_product_never_imports_the_oracle():
    """The package, the bench's GPU leg and the build step contain no reference to oracle/ (only the
    cpu_baseline function of bench.py and the smoke check do)."""
    pkg = os.path.join(ROOT, "paper_2601_07876_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    bench = open(os.path.join(ROOT, "bench.py")).read()
    body = bench.split("def cpu_baseline(")[0] + bench.split("def main():")[1]
    assert "from oracle" not in body and "import oracle" not in body


@pytest.mark.parametrize("name", ["ragged", "c2_resnet50", "c4_vit_b16_bf16", "c5_decoder_1p3b"])
def test_arena_plan_places_every_tensor_on_its_own_aligned_range(name):
    numels = W.get_workload(name).numels
    rc, offs, role_elems, stride = N.novak_plan_arena(numels)
    assert rc == N.NOVAK_OK
    end = 0
    for o, n in zip(offs, numels):
        assert o % 256 == 0 and o >= end          # 1 KB-aligned for 4-byte elements, no overlap, tensor order kept
        end = o + n
    assert role_elems >= end and role_elems % 256 == 0 and role_elems - end < 256
    assert stride >= role_elems * 4 and stride % 8192 == 2048 and stride - role_elems * 4 < 8192 + 2048


def test_arena_plan_edge_cases():
    assert N.novak_plan_arena([]) == (N.NOVAK_OK, [], 0, 2048)
    assert N.novak_plan_arena([0, 0]) == (N.NOVAK_OK, [0, 0], 0, 2048)
    assert N.novak_plan_arena([1]) == (N.NOVAK_OK, [0], 256, 8192 + 2048)
    assert N.novak_plan_arena([2048, 1])[1:] == ([0, 2048], 2304, 16384 + 2048)
    assert N.novak_plan_arena([-1])[0] == N.NOVAK_ERR_INVALID_ARG
    assert N.novak_plan_arena([2 ** 62, 2 ** 62])[0] == N.NOVAK_ERR_INVALID_ARG
    lib = N.load_library()
    i64 = C.c_int64
    arr, a, b = (i64 * 2)(5, 7), i64(0), i64(0)
    assert lib.novak_plan_arena(arr, 2, None, C.byref(a), C.byref(b)) == N.NOVAK_OK and a.value == 512   # offsets optional
    assert lib.novak_plan_arena(arr, 2, None, None, C.byref(b)) == N.NOVAK_ERR_NULL_POINTER
    assert lib.novak_plan_arena(None, 2, None, C.byref(a), C.byref(b)) == N.NOVAK_ERR_NULL_POINTER
    assert lib.novak_plan_arena(arr, -1, None, C.byref(a), C.byref(b)) == N.NOVAK_ERR_INVALID_ARG
