"""Test-side plumbing: runs the HIP path through the C ABI and the oracle on the same inputs.

Holds no optimizer arithmetic.  The GPU side only allocates torch tensors, hands raw pointers to the
library and copies results back; the oracle side calls oracle/novak_oracle.py.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N

LA_NAMES = {0: "none", 1: "memory_efficient", 2: "basic"}
NEST_NAMES = {0: "none", 1: "approx", 2: "classical", 3: "true"}
MOMENT_NAMES = {0: "f32", 1: "bf16_m"}

# the parity bound of the benchmark spec: |gpu - ref| <= 1e-7 + 1e-5 |ref|, per element
ATOL, RTOL = 1e-7, 1e-5


def oracle_hyper(hyper: Dict[str, object], effective_nesterov: Optional[str] = None,
                 effective_lookahead: Optional[str] = None, info=None) -> O.Hyper:
    """Oracle hyper-parameters for what the library says it effectively runs (after fast-path downgrades)."""
    h = {k: v for k, v in hyper.items() if k not in ("mode", "auto_sync")}
    if effective_nesterov is not None:
        h["nesterov"] = effective_nesterov
    if effective_lookahead is not None:
        h["lookahead"] = effective_lookahead
    if info is not None:
        h["layer_adaptation"] = bool(info.layer_adaptation)
        h["auto_lr"] = bool(info.auto_lr)
        h["use_gc"] = bool(info.use_gc)
        h["moment_dtype"] = MOMENT_NAMES[info.moment_dtype]
    return O.Hyper(**h)


class GpuNovak:
    """Device buffers for a tensor list plus a library handle.

    `misalign` shifts every state tensor by that many elements inside its allocation (to leave the
    16-byte path); `guard` adds that many sentinel elements on both sides of every tensor.
    """
    SENTINEL = 12288.0      # exactly representable in bfloat16 too

    def __init__(self, numels: Sequence[int], hyper: Dict[str, object], grad_dtype: str = "f32",
                 theta0: Optional[List[np.ndarray]] = None, misalign: int = 0, guard: int = 0,
                 chunk_elems: Optional[int] = None, nontemporal: Optional[bool] = None,
                 auto_sync: bool = False, device: str = "cuda:0", lookahead_init: bool = True,
                 vec_per_lane: Optional[int] = None, threads: Optional[int] = None, rows: Optional[Sequence[int]] = None):
        self.numels = list(numels)
        self.rows = list(rows) if rows is not None else [0] * len(self.numels)
        self.hyper = dict(hyper)
        self.grad_dtype = grad_dtype
        self.device = torch.device(device)
        self.guard, self.misalign = guard, misalign
        self.pad = guard + misalign
        self._raw = {}
        self.theta, self.m, self.v, self.la = [], [], [], []
        m_dtype = torch.bfloat16 if self.hyper.get("moment_dtype", "f32") == "bf16_m" else torch.float32
        for i, n in enumerate(self.numels):
            for role, lst in (("theta", self.theta), ("m", self.m), ("v", self.v), ("la", self.la)):
                raw = torch.full((n + 2 * self.pad + 4,), self.SENTINEL, dtype=m_dtype if role == "m" else torch.float32,
                                 device=self.device)
                view = raw[self.pad: self.pad + n]
                self._raw[(role, i)] = raw
                lst.append(view)
            self.m[i].zero_()
            self.v[i].zero_()
            if theta0 is not None:
                self.theta[i].copy_(torch.from_numpy(np.ascontiguousarray(theta0[i], dtype=np.float32)))
        hp = N.make_hparams(auto_sync=auto_sync, **self.hyper)
        descs = [N.novak_tensor_desc(self.theta[i].data_ptr(), self.m[i].data_ptr(), self.v[i].data_ptr(),
                                     self.la[i].data_ptr(), n, self.rows[i]) for i, n in enumerate(self.numels)]
        rc, self.handle = N.novak_create(hp, descs, self.device.index or 0)
        N.check(rc, "novak_create")
        if chunk_elems is not None:
            N.check(N.novak_set_tuning(self.handle, N.NOVAK_TUNE_CHUNK_ELEMS, chunk_elems), "set_tuning", self.handle)
        if nontemporal is not None:
            N.check(N.novak_set_tuning(self.handle, N.NOVAK_TUNE_NONTEMPORAL, int(nontemporal)), "set_tuning", self.handle)
        if vec_per_lane is not None:
            N.check(N.novak_set_tuning(self.handle, N.NOVAK_TUNE_VEC_PER_LANE, vec_per_lane), "set_tuning", self.handle)
        if threads is not None:
            N.check(N.novak_set_tuning(self.handle, N.NOVAK_TUNE_THREADS, threads), "set_tuning", self.handle)
        rc, info = N.novak_get_info(self.handle)
        N.check(rc, "novak_get_info", self.handle)
        self.info = info
        self.eff_lookahead = LA_NAMES[info.lookahead_mode]
        self.eff_nesterov = NEST_NAMES[info.nesterov_mode]
        self.auto_sync = auto_sync
        self.la_k = int(self.hyper.get("la_k", 5))
        self._grad_arr = (C.c_void_p * max(len(self.numels), 1))()
        self.ema = None
        if info.auto_lr:
            self.ema = torch.zeros(2, dtype=torch.float64, device=self.device)
            N.check(N.novak_set_auto_lr_state(self.handle, self.ema.data_ptr()), "novak_set_auto_lr_state", self.handle)
        if lookahead_init and self.eff_lookahead != "none":
            N.check(N.novak_lookahead_init(self.handle, self.stream), "novak_lookahead_init", self.handle)

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def upload_grads(self, grads_host: List[np.ndarray], misalign: int = 0) -> List[torch.Tensor]:
        """Host fp32 gradient values -> device tensors of the run's gradient dtype."""
        out = []
        for g in grads_host:
            t = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32))
            if self.grad_dtype == "bf16":
                t = t.to(torch.bfloat16)     # exact: values were rounded to bf16 by the generator
            raw = torch.empty(t.numel() + misalign + 8, dtype=t.dtype, device=self.device)
            view = raw[misalign: misalign + t.numel()]
            view.copy_(t)
            out.append(view)
        return out

    def step(self, t: int, grads: List[torch.Tensor], sync: bool = True) -> int:
        for i, g in enumerate(grads):
            self._grad_arr[i] = g.data_ptr() if g.numel() else None
        rc = N.novak_step(self.handle, self._grad_arr, N.GRAD_DTYPE[self.grad_dtype], t, self.stream)
        if rc != N.NOVAK_OK:
            return rc
        if sync and not self.auto_sync and self.eff_lookahead != "none" and t % self.la_k == 0:
            rc = N.novak_lookahead_sync(self.handle, self.stream)
        return rc

    def host(self, role: str) -> List[np.ndarray]:
        torch.cuda.synchronize(self.device)
        return [x.detach().float().cpu().numpy().copy() for x in getattr(self, role)]

    def tensor_scales(self) -> np.ndarray:
        """lambda_trust * alpha_auto per tensor of the last two-pass step."""
        rc, vals = N.novak_copy_tensor_scales(self.handle, len(self.numels), self.stream)
        N.check(rc, "novak_copy_tensor_scales", self.handle)
        return np.array(vals, dtype=np.float64)

    def guards_intact(self) -> bool:
        torch.cuda.synchronize(self.device)
        for (role, i), raw in self._raw.items():
            n = self.numels[i]
            left, right = raw[: self.pad], raw[self.pad + n:]
            if not bool((left == self.SENTINEL).all()) or not bool((right == self.SENTINEL).all()):
                return False
        return True

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            N.novak_destroy(self.handle)
            self.handle = None


def assert_close(name: str, got: np.ndarray, ref: np.ndarray, atol: float = ATOL, rtol: float = RTOL):
    got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
    err = np.abs(got64 - ref64)
    bound = atol + rtol * np.abs(ref64)
    bad = ~(err <= bound)
    if bad.any():
        j = int(np.argmax(err - bound))
        raise AssertionError(f"{name}: {int(bad.sum())}/{bad.size} elements outside |d| <= {atol} + {rtol}|ref|; "
                             f"worst at {j}: got {got64[j]!r} ref {ref64[j]!r} err {err[j]:.3e}")


def assert_close_strict(name: str, got: np.ndarray, ref: np.ndarray, rtol: float = 2e-6):
    """Tighter, scale-aware check: |d| <= rtol * (|ref| + rms(ref)).  Keeps m and v meaningful even
    where the benchmark's absolute floor of 1e-7 exceeds their magnitude."""
    got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
    scale = float(np.sqrt(np.mean(ref64 * ref64))) if ref64.size else 0.0
    err = np.abs(got64 - ref64)
    bound = rtol * (np.abs(ref64) + scale) + 1e-38
    bad = ~(err <= bound)
    if bad.any():
        j = int(np.argmax(err - bound))
        raise AssertionError(f"{name} (strict): {int(bad.sum())}/{bad.size} outside; worst at {j}: "
                             f"got {got64[j]!r} ref {ref64[j]!r} err {err[j]:.3e} bound {bound[j]:.3e}")


def run_pair(numels: Sequence[int], hyper: Dict[str, object], steps: int, grad_std: float, grad_dtype: str = "f32",
             seed: int = 42, auto_sync: bool = False, chunk_elems: Optional[int] = None,
             nontemporal: Optional[bool] = None, misalign: int = 0, grad_misalign: int = 0, guard: int = 0,
             check_blend_at: Sequence[int] = (), vec_per_lane: Optional[int] = None, threads: Optional[int] = None,
             rows: Optional[Sequence[int]] = None):
    """Runs GPU and oracle over host-generated inputs; returns (gpu, oracle states) after `steps`."""
    theta0 = W.host_params(numels, seed)
    gpu = GpuNovak(numels, hyper, grad_dtype, theta0, misalign=misalign, guard=guard, chunk_elems=chunk_elems,
                   nontemporal=nontemporal, auto_sync=auto_sync, vec_per_lane=vec_per_lane, threads=threads, rows=rows)
    h = oracle_hyper(hyper, gpu.eff_nesterov, gpu.eff_lookahead, gpu.info)
    states = [O.init_state(th, h, rows=gpu.rows[i]) for i, th in enumerate(theta0)]
    aux = O.AutoLrState()
    for t in range(1, steps + 1):
        gh = W.host_grads(numels, t, grad_std, seed, bf16=(grad_dtype == "bf16"))
        gd = gpu.upload_grads(gh, misalign=grad_misalign)
        N.check(gpu.step(t, gd), f"novak_step t={t}", gpu.handle)
        O.step_all(states, gh, t, h, aux)
        if t in check_blend_at and h.lookahead == "memory_efficient" and not (auto_sync and t % h.la_k == 0):
            la = gpu.host("la")
            for i, st in enumerate(states):
                keep = slice(None) if st.ambiguous is None else ~st.ambiguous
                assert_close(f"la_buf[{i}] t={t}", la[i][keep], O.blend_buffer(st, h)[keep])
        if O.sync_due(t, h):
            for st in states:
                O.lookahead_sync(st, h)
    return gpu, states, h


def split_ambiguous(name: str, got: np.ndarray, ref: np.ndarray, ambiguous: Optional[np.ndarray], max_move: float,
                    max_fraction: float = 2e-3):
    """Elements for which a discontinuous decision (the Eq. 27 mask, the bfloat16 rounding of a stored
    moment) was within fp32 rounding of its threshold at some step may legitimately differ by up to the
    steps they took or skipped, or by a few bfloat16 ulps: they are checked against that weaker bound
    and removed from the element-wise comparison.  Their fraction must stay small."""
    if ambiguous is None or not ambiguous.any():
        return got, ref
    count = int(ambiguous.sum())
    expected = max_fraction * ambiguous.size
    assert count <= expected + 3.0 * expected ** 0.5 + 2.0, \
        f"{name}: {count}/{ambiguous.size} elements are ambiguous - the band is too wide to mean anything"
    d = np.abs(got[ambiguous].astype(np.float64) - ref[ambiguous].astype(np.float64))
    assert np.all(d <= max_move), f"{name}: an ambiguous element moved by {d.max():.3e} > {max_move:.3e}"
    keep = ~ambiguous
    return got[keep], ref[keep]


def compare_states(gpu: GpuNovak, states: List[O.TensorState], strict: bool = True, tag: str = "", max_move: float = 2e-2,
                   max_fraction: float = 2e-3):
    """`max_move` bounds how far an element with an ambiguous decision may sit from the oracle's theta.

    With the first moment stored in bfloat16 the flagged elements' m and v are held to a few bf16 ulps
    of the tensor's largest |m| (a one-ulp difference in m persists and feeds v through Eq. 13), and
    every other element's m must be bit-identical to the oracle's."""
    th, m, v = gpu.host("theta"), gpu.host("m"), gpu.host("v")
    bf16_m = gpu.hyper.get("moment_dtype", "f32") == "bf16_m"
    for i, st in enumerate(states):
        th_i, ref_i = split_ambiguous(f"{tag}theta[{i}]", th[i], st.theta, st.ambiguous, max_move, max_fraction)
        assert_close(f"{tag}theta[{i}]", th_i, ref_i)
        if strict and ref_i.size:
            assert_close_strict(f"{tag}theta[{i}]", th_i, ref_i)
        m_i, mref_i, v_i, vref_i = m[i], st.m, v[i], st.v
        if bf16_m and st.m.size:
            m_i, mref_i = split_ambiguous(f"{tag}m[{i}]", m[i], st.m, st.ambiguous, 2.0 ** -5 * float(np.abs(st.m).max()), max_fraction)
            v_i, vref_i = split_ambiguous(f"{tag}v[{i}]", v[i], st.v, st.ambiguous, 2.0 ** -5 * float(np.abs(st.v).max()), max_fraction)
            assert np.array_equal(m_i, mref_i), f"{tag}m[{i}]: bfloat16 first moment differs on {int((m_i != mref_i).sum())} unflagged elements"
        assert_close(f"{tag}m[{i}]", m_i, mref_i)
        assert_close(f"{tag}v[{i}]", v_i, vref_i)
        if strict and mref_i.size:
            assert_close_strict(f"{tag}m[{i}]", m_i, mref_i)
            assert_close_strict(f"{tag}v[{i}]", v_i, vref_i)
