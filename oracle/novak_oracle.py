"""CPU oracle of the NOVAK per-parameter update step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, by-eye-checkable statement of what one optimizer step computes, written from the
paper's equations (section 4, Eq. 1-31; the ten-phase order of section 5.1 and Table 2).  It shares
no code with the HIP path.  Nothing in the product may import it: only tests, the smoke check and
the benchmark's cpu_baseline leg do.

Arithmetic is IEEE double throughout.  `state_dtype=np.float32` (the default) rounds theta, m, v and
the slow weights to fp32 once at the end of every step / sync, which is what "fp32 steps" means;
`state_dtype=np.float64` gives the all-double trajectory used to separate algorithm from rounding.

Readings taken where the paper is silent or inconsistent (each is a named switch or stated here):
  * unrect_fallback: what the step is while rho_t < 5 (Eq. 8 only gives alpha_eff = alpha/(1-beta1^t)
    and never says the sqrt(v_hat) denominator is dropped).  "adam_denom" keeps the denominator with
    r_t = 1 (the paper's Eq. 24 taken literally); "sgdm" drops it (theta -= alpha*m_hat, the original
    RAdam behaviour).
  * The 1/(1-beta1^t) of Eq. 8 and the m_hat of Eq. 24 are the same bias correction; applied once.
  * Lookahead "memory_efficient": slow_new = slow_0 + alpha_LA * (1/k) * sum_{i=1..k}(theta_i - slow_0),
    the mean over ALL k fast iterates of the window (Theorem 6.2 proof, text under Eq. 29, section
    7.2).  The literal Eq. 29 (sum of negated single-step updates) contradicts Eq. 30's 1/k and the
    four restatements, and is not used.  "basic" is standard Lookahead: slow_0 + alpha_LA*(theta_k - slow_0).
  * Sync happens after the steps with t mod k == 0, t counted from 1; the window starts at theta_0.
    A sync does not touch m or v.
  * decoupled_decay = False is listed by the paper with no formula; read as classic coupled L2,
    g <- g + lambda*theta before everything else.  parity unpinned by the paper (pinned only against
    torch.optim.Adam's weight_decay semantics).
  * beta_n has no default in the paper.  parity unpinned by the paper for its value; callers pass it.
  * nesterov "true": the gradient handed in is already the one evaluated at the extrapolated point
    (Eq. 10-11 need a model); the moment pipeline of Eq. 24 then runs as for "none".
  * nesterov "classical": Eq. 16 literally (blend of un-normalised m_hat with the normalised u).
  * layer adaptation (Eq. 19 / 25), per tensor: eta = ||theta||_2 / ||u||_2 with theta the parameters
    BEFORE this step's decay/update and u the base direction of Eq. 17 (Table 2 computes the ratio in
    Phase 7, before the classical blend of Phase 8); clipped to [0.1, 10]; eta = 1 when either norm is
    zero (LAMB's convention; the paper is silent).  parity unpinned by the paper for these choices.
  * auto-LR (Eq. 20-22): EMAs (gamma = 0.1, started at 0) of the GLOBAL norms over all tensors (Table 3
    stores two scalars), of the gradient as handed in and of the parameters before the step;
    alpha_auto = clip(g_bar / theta_bar, 0.1, 2), and 1 when theta_bar is 0.  Eq. 23 is a second,
    different formula for the same symbol that the paper calls an alternative; it is not used.
    parity unpinned by the paper for scope, initial value and the gradient's processing stage.
  * alpha_eff = alpha * r_t * eta_clipped * alpha_auto (Eq. 24a); the decay keeps the base alpha.
  * gradient clipping (sections 5.8, 7.3; Table 2 Phase 2): if the GLOBAL norm over all tensors of the
    gradient as handed in exceeds c_clip, every gradient is scaled by c_clip/norm, before any other
    processing (coupled decay, Nesterov approximation).  The auto-LR norm of Eq. 20 keeps using the
    gradient as handed in.  parity unpinned by the paper for that last choice.
  * gradient centralization (Eq. 26; full-features mode, tensors with more than one dimension): the
    mean over all dimensions but the first is subtracted from each dim-0 slice.  It runs after the
    clipping and before the Nesterov approximation (section 7.3 puts clipping before any other
    processing; Table 2 lists the approximation last in Phase 2).  A tensor opts in through
    TensorState.rows = size of its first dimension (0 = not centralized).
  * adaptive beta (Eq. 3-4): beta_i(t) = beta_i * (1 - exp(-t/tau_i)) replaces beta_i in the moment
    updates (Eq. 1-2) at every t (the schedule is smooth and asymptotic; the text's "t < tau_1" is read
    as describing where it matters, not a cut-off).  Bias correction (Eq. 5), the rectification
    schedule (Eq. 6-9) and the classical blend (Eq. 16) keep the base betas, as printed.
    parity unpinned by the paper for this interplay.
  * true Nesterov (Eq. 10): the extrapolated point is theta + beta_n * m with the sign as printed;
    `extrapolate` returns it.  With n_taylor > 0 the mode "true" behaves as "approx" for t > n_taylor
    (automatic fallback, sections 4.4 and 5.8).
  * reduced-precision first moment (the paper's "multi-precision" outlook, sections 3 and 10.3; not part
    of its method): moment_dtype = "bf16_m" stores m as bfloat16, rounded to nearest-even from the
    exactly computed value of Eq. 1; that stored m_t is what bias correction and the direction of the
    same step use.  All arithmetic stays in double here (fp32 in an implementation).  v stays fp32: with
    beta2 = 0.999 its per-step change (0.1 % of v) is below half a bfloat16 ulp (0.2-0.4 %), so a
    round-to-nearest bf16 v would stop moving.  The rounding is a discontinuous decision: an
    implementation that forms m in fp32 can land on the other side of a rounding boundary.  The oracle
    does not model that; it exposes the exact m_t before the rounding (TensorState.trace) and accepts,
    through `stored_m`, the value an implementation stored, so that a comparison can check the rounding
    itself and then the rest of the step given that rounding.  parity unpinned by the paper (it defines
    no such mode).
  * sparse threshold (Eq. 27): the base direction u is zeroed where |u| <= tau, after the trust ratio is
    taken (Phase 7 precedes Phase 8) and before the classical blend (Table 2's order within Phase 8).
    The mask is a discontinuous decision on a floating-point value: an implementation in another
    precision may decide differently where |u| is within rounding of tau.  The oracle does not model
    that either; it exposes |u| before the mask (TensorState.trace) for comparisons to judge.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

NESTEROV_MODES = ("none", "approx", "classical", "true")
LOOKAHEAD_MODES = ("none", "memory_efficient", "basic")
UNRECT_FALLBACKS = ("adam_denom", "sgdm")
MOMENT_DTYPES = ("f32", "bf16_m")


@dataclass
class Hyper:
    """Hyper-parameters of Algorithm 1's header (section 5.2)."""
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    beta_n: float = 0.9
    la_alpha: float = 0.5
    la_k: int = 5
    rectified: bool = True
    decoupled_decay: bool = True
    nesterov: str = "approx"
    lookahead: str = "memory_efficient"
    unrect_fallback: str = "adam_denom"
    layer_adaptation: bool = False      # Eq. 19 / 25 (full-features mode)
    auto_lr: bool = False               # Eq. 20-22 (full-features mode)
    auto_lr_gamma: float = 0.1
    trust_clip: tuple = (0.1, 10.0)
    auto_clip: tuple = (0.1, 2.0)
    clip_threshold: float = 0.0         # c_clip on the global gradient norm; 0 = off (section 5.8)
    sparse_threshold: float = 0.0       # tau of Eq. 27; 0 = off
    use_gc: bool = False                # Eq. 26 on tensors that declare rows >= 1
    adaptive_beta: bool = False         # Eq. 3-4
    beta_tau1: float = 1000.0
    beta_tau2: float = 5000.0
    n_taylor: int = 0                   # "true" Nesterov falls back to "approx" after this many steps; 0 = never
    moment_dtype: str = "f32"           # "bf16_m": m is stored as bfloat16 (see header)

    def __post_init__(self):
        assert self.nesterov in NESTEROV_MODES
        assert self.lookahead in LOOKAHEAD_MODES
        assert self.unrect_fallback in UNRECT_FALLBACKS
        assert self.moment_dtype in MOMENT_DTYPES


@dataclass
class StepScalars:
    """Per-step scalars shared by every element (Phases 5-6)."""
    bc1: float          # 1 - beta1^t            (Eq. 5)
    bc2: float          # 1 - beta2^t            (Eq. 5)
    rho_inf: float      # Eq. 6
    rho_t: float        # Eq. 7
    rectified_now: bool  # rho_t >= 5 and rectification enabled
    r_t: float          # Eq. 9, or 1 when not rectified_now
    denom_on: bool      # whether u carries the sqrt(v_hat)+eps denominator
    step_size: float    # alpha * r_t            (Eq. 24a with lambda_trust = alpha_auto = 1)
    decay: float        # 1 - alpha*lambda       (Eq. 18), or 1 when decay is coupled


def one_minus_pow(beta: float, t: int) -> float:
    """1 - beta^t, through the logarithm as section 5.8 prescribes: 1 - exp(t*log(beta))."""
    if beta == 0.0:
        return 1.0
    return -math.expm1(t * math.log(beta))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round double values to the nearest bfloat16 (8 significant bits, ties to even) in ONE rounding.

    Returns the rounded values as float64.  Subnormal bfloat16 results are not handled (the moments
    here never get below 1e-38).
    """
    x = np.asarray(x, dtype=np.float64)
    mant, exp = np.frexp(x)                      # x = mant * 2^exp, 0.5 <= |mant| < 1
    q = np.rint(mant * 256.0)                    # 128 <= |mant * 256| < 256: one unit = one bf16 ulp; ties to even
    return np.ldexp(q, exp - 8)


def scheduled_betas(h: Hyper, t: int):
    """(beta1, beta2) used by the moment updates at step t (Eq. 3-4 when adaptive_beta, else the base values)."""
    if not h.adaptive_beta:
        return h.beta1, h.beta2
    return (h.beta1 * (1.0 - math.exp(-t / h.beta_tau1)),      # Eq. 3
            h.beta2 * (1.0 - math.exp(-t / h.beta_tau2)))      # Eq. 4


def effective_nesterov(h: Hyper, t: int) -> str:
    """Nesterov variant in force at step t: "true" hands over to "approx" after n_taylor steps."""
    if h.nesterov == "true" and h.n_taylor > 0 and t > h.n_taylor:
        return "approx"
    return h.nesterov


def extrapolate(st: "TensorState", h: Hyper) -> np.ndarray:
    """Eq. 10: the point at which true Nesterov evaluates the gradient (double)."""
    return st.theta.astype(np.float64) + h.beta_n * st.m.astype(np.float64)


def step_scalars(h: Hyper, t: int) -> StepScalars:
    """Scalars of step t (t = 1 on the first step; Eq. 5 is undefined at t = 0)."""
    assert t >= 1
    bc1 = one_minus_pow(h.beta1, t)
    bc2 = one_minus_pow(h.beta2, t)
    rho_inf = 2.0 / (1.0 - h.beta2) - 1.0                                  # Eq. 6
    beta2_t = 1.0 - bc2
    rho_t = rho_inf - 2.0 * t * beta2_t / bc2                              # Eq. 7
    r_t, rect_now, denom_on = 1.0, False, True
    if h.rectified:
        if rho_t >= 5.0:                                                   # Eq. 8, first case
            rect_now = True
            r_t = math.sqrt((rho_t - 4.0) * (rho_t - 2.0) * rho_inf /
                            ((rho_inf - 4.0) * (rho_inf - 2.0) * rho_t))   # Eq. 9
        else:                                                              # Eq. 8, second case
            denom_on = (h.unrect_fallback == "adam_denom")
    decay = 1.0 - h.lr * h.weight_decay if h.decoupled_decay else 1.0      # Eq. 18
    return StepScalars(bc1, bc2, rho_inf, rho_t, rect_now, r_t, denom_on, h.lr * r_t, decay)


@dataclass
class StepTrace:
    """Intermediate values of a tensor's most recent step, kept for comparisons (they change no result)."""
    g_processed: np.ndarray      # the gradient after clipping, centralization and coupled decay, before Eq. 13
    g_terms: np.ndarray          # |scaled g| + |row mean| + lambda |theta|: magnitudes of the terms g_processed is made of
    g_tilde: np.ndarray          # the gradient that fed the moments (Eq. 13 applied when in force)
    m_exact: np.ndarray          # Eq. 1 in double, before any storage rounding
    u_base: np.ndarray           # base direction of Eq. 17 (or m_hat in the momentum fallback), before Eq. 27 / Eq. 16
    scale: float                 # lambda_trust * alpha_auto of Eq. 24a


@dataclass
class TensorState:
    """State of one parameter tensor (Table 3): theta, m, v and the lookahead window."""
    theta: np.ndarray
    m: np.ndarray
    v: np.ndarray
    slow0: Optional[np.ndarray] = None                 # theta_0^slow of the open window (Eq. 28)
    window: List[np.ndarray] = field(default_factory=list)   # the fast iterates of the open window
    rows: int = 0                                      # size of dim 0 if the tensor has more than one dim, else 0 (Eq. 26)
    trace: Optional[StepTrace] = None                  # see StepTrace

    @property
    def dtype(self):
        return self.theta.dtype


def init_state(theta0: np.ndarray, h: Hyper, state_dtype=np.float32, rows: int = 0) -> TensorState:
    """m_0 = v_0 = 0; with lookahead on, slow weights start at theta_0 (Eq. 28, section 5.8)."""
    theta = np.array(theta0, dtype=state_dtype).reshape(-1).copy()
    st = TensorState(theta, np.zeros_like(theta), np.zeros_like(theta), rows=rows)
    if h.lookahead != "none":
        st.slow0 = theta.copy()
    return st


def trust_ratio(theta: np.ndarray, u: np.ndarray, h: Hyper) -> float:
    """Clipped layer-wise trust ratio of one tensor (Eq. 19, Eq. 25)."""
    n_theta = math.sqrt(float(np.dot(theta, theta)))
    n_u = math.sqrt(float(np.dot(u, u)))
    eta = n_theta / n_u if (n_theta > 0.0 and n_u > 0.0) else 1.0
    return min(max(eta, h.trust_clip[0]), h.trust_clip[1])


@dataclass
class AutoLrState:
    """The two scalars of Table 3: EMAs of the gradient norm and the parameter norm (Eq. 20-21)."""
    g_bar: float = 0.0
    theta_bar: float = 0.0


def auto_lr_scale(aux: AutoLrState, thetas, grads, h: Hyper) -> float:
    """Updates the EMAs from the global norms (Eq. 20-21) and returns alpha_auto (Eq. 22)."""
    g2 = sum(float(np.dot(x, x)) for x in (np.asarray(g, dtype=np.float64).reshape(-1) for g in grads))
    t2 = sum(float(np.dot(x, x)) for x in (np.asarray(th, dtype=np.float64).reshape(-1) for th in thetas))
    gam = h.auto_lr_gamma
    aux.g_bar = gam * math.sqrt(g2) + (1.0 - gam) * aux.g_bar          # Eq. 20
    aux.theta_bar = gam * math.sqrt(t2) + (1.0 - gam) * aux.theta_bar  # Eq. 21
    if aux.theta_bar == 0.0:
        return 1.0
    return min(max(aux.g_bar / aux.theta_bar, h.auto_clip[0]), h.auto_clip[1])   # Eq. 22


def clip_scale(grads, h: Hyper) -> float:
    """Factor applied to every gradient: c_clip/||g|| when the global norm exceeds c_clip, else 1."""
    if h.clip_threshold <= 0.0:
        return 1.0
    g2 = sum(float(np.dot(x, x)) for x in (np.asarray(g, dtype=np.float64).reshape(-1) for g in grads))
    norm = math.sqrt(g2)
    return h.clip_threshold / norm if norm > h.clip_threshold else 1.0


def step(st: TensorState, grad: np.ndarray, t: int, h: Hyper, alpha_auto: float = 1.0,
         g_scale: float = 1.0, stored_m: Optional[np.ndarray] = None) -> StepScalars:
    """One update of one tensor at step t (Phases 2-9), then record the iterate for lookahead.

    `grad` holds the gradient values (any float dtype; bf16 gradients arrive as the fp32/fp64
    numbers they exactly represent).  The sync of Phase 10 is a separate call: `lookahead_sync`.
    `alpha_auto` is the step-wide auto-LR factor (1 unless h.auto_lr; see `auto_lr_scale`);
    `g_scale` the step-wide clipping factor (see `clip_scale`).
    `stored_m` (moment_dtype "bf16_m" only; for comparisons): the bfloat16 values an implementation
    stored as m_t.  When given they stand in for the oracle's own rounding of the exact m_t in the rest
    of the step; whether they are a legitimate rounding of st.trace.m_exact is for the caller to check.
    """
    s = step_scalars(h, t)
    dt = st.dtype
    theta = st.theta.astype(np.float64)
    m_prev = st.m.astype(np.float64)
    v_prev = st.v.astype(np.float64)
    g = np.asarray(grad).reshape(-1).astype(np.float64) * g_scale   # clipping comes first (section 7.3)
    g_terms = np.abs(g)

    if h.use_gc and st.rows >= 1:
        g2d = g.reshape(st.rows, -1)
        row_mean = g2d.mean(axis=1, keepdims=True)
        g = (g2d - row_mean).reshape(-1)                    # Eq. 26
        g_terms = g_terms + np.broadcast_to(np.abs(row_mean), g2d.shape).reshape(-1)
    if (not h.decoupled_decay) and h.weight_decay != 0.0:
        g = g + h.weight_decay * theta                      # coupled L2 (reading; see header)
        g_terms = g_terms + h.weight_decay * np.abs(theta)
    g_processed = g
    if effective_nesterov(h, t) == "approx":
        g = g + h.beta_n * (g - m_prev)                     # Eq. 13; replaces g for both moments
    b1_t, b2_t = scheduled_betas(h, t)                      # Eq. 3-4 (Phase 3)
    m = b1_t * m_prev + (1.0 - b1_t) * g                    # Eq. 1
    v = b2_t * v_prev + (1.0 - b2_t) * g * g                # Eq. 2
    m_exact = m
    if h.moment_dtype == "bf16_m":                          # m_t is what is stored: the rest of the step uses it
        m = round_to_bf16(m_exact) if stored_m is None else np.asarray(stored_m, dtype=np.float64).reshape(-1)
    else:
        assert stored_m is None
    m_hat = m / s.bc1                                       # Eq. 5
    if s.denom_on:
        v_hat = v / s.bc2                                   # Eq. 5
        u = m_hat / (np.sqrt(v_hat) + h.eps)                # Eq. 17
    else:
        u = m_hat                                           # momentum-SGD fallback while rho_t < 5
    u_base = u
    lam_trust = trust_ratio(theta, u, h) if h.layer_adaptation else 1.0   # Eq. 19 / 25 (Phase 7)
    if h.sparse_threshold > 0.0:
        u = np.where(np.abs(u) > h.sparse_threshold, u, 0.0)   # Eq. 27
    if h.nesterov == "classical":
        u = h.beta1 * m_hat + (1.0 - h.beta1) * u           # Eq. 16
    alpha_eff = s.step_size * lam_trust * alpha_auto        # Eq. 24a
    theta = theta * s.decay - alpha_eff * u                 # Eq. 18 then Eq. 24

    st.theta = theta.astype(dt)
    st.m = m.astype(dt)
    st.v = v.astype(dt)
    st.trace = StepTrace(g_processed, g_terms, g, m_exact, u_base, lam_trust * alpha_auto)
    if h.lookahead != "none":
        st.window.append(st.theta.copy())
    return s


def sync_due(t: int, h: Hyper) -> bool:
    """Phase 10: synchronise after the steps with t mod k == 0."""
    return h.lookahead != "none" and t % h.la_k == 0


def lookahead_sync(st: TensorState, h: Hyper) -> None:
    """Eq. 30-31 at the end of a k-step window, from the stored iterates (the plain definition)."""
    assert h.lookahead != "none"
    assert len(st.window) == h.la_k, "sync is defined at the end of a full window"
    slow0 = st.slow0.astype(np.float64)
    if h.lookahead == "memory_efficient":
        delta = np.zeros_like(slow0)
        for th in st.window:                                # Delta = sum_i (theta_i - slow_0)
            delta += th.astype(np.float64) - slow0
        slow_new = slow0 + h.la_alpha * delta / h.la_k      # Eq. 30
    else:                                                   # "basic": standard Lookahead
        slow_new = slow0 + h.la_alpha * (st.window[-1].astype(np.float64) - slow0)
    st.theta = slow_new.astype(st.dtype)                    # Eq. 31
    st.slow0 = st.theta.copy()                              # new reference point, Delta reset
    st.window = []


def step_all(states: List[TensorState], grads, t: int, h: Hyper, aux: Optional[AutoLrState] = None,
             stored_m: Optional[list] = None) -> float:
    """One step over a tensor list: the step-wide auto-LR factor first (Phase 7), then every tensor.

    Returns alpha_auto; every tensor's lambda_trust * alpha_auto is left in its trace.  `stored_m`:
    one entry per tensor, see `step`."""
    alpha_auto = 1.0
    if h.auto_lr:
        assert aux is not None, "auto_lr needs its two EMA scalars"
        alpha_auto = auto_lr_scale(aux, [st.theta for st in states], grads, h)
    g_scale = clip_scale(grads, h)
    for i, (st, g) in enumerate(zip(states, grads)):
        step(st, g, t, h, alpha_auto, g_scale, None if stored_m is None else stored_m[i])
    return alpha_auto


def run(theta0_list, grads_fn, steps: int, h: Hyper, state_dtype=np.float32, t0: int = 0,
        states: Optional[List[TensorState]] = None, aux: Optional[AutoLrState] = None,
        rows: Optional[List[int]] = None) -> List[TensorState]:
    """Run `steps` steps over a list of tensors; grads_fn(t) returns the gradient list of step t."""
    if states is None:
        states = [init_state(th, h, state_dtype, rows[i] if rows else 0) for i, th in enumerate(theta0_list)]
    if aux is None:
        aux = AutoLrState()
    for t in range(t0 + 1, t0 + steps + 1):
        grads = grads_fn(t)
        step_all(states, grads, t, h, aux)
        if sync_due(t, h):
            for st in states:
                lookahead_sync(st, h)
    return states
