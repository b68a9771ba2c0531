"""Seeded synthetic inputs for the MoE-layer hot path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds no arithmetic of the method itself (no gate, no routing,
no FFN): it only draws random tensors with the shapes of the paper's evaluation
models (Table 1: BERT/GPT/Swin MoE layers), encodes a per-expert logit bias that
reproduces the skewed expert loads reported in the paper's load trace
(Observation 2: ten of 64 experts receive about three quarters of the tokens,
and the hot set drifts smoothly), and builds expert->vExpert placement tables
from a vector of per-expert loads.

bf16 tensors are kept as uint16 bit patterns so that every consumer sees the
same rounded values; `Bf16Tensor` decodes slices to float32 on demand.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 230403946

ACT_RELU, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2
DT_F32, DT_BF16 = 0, 1


# ----------------------------------------------------------------------------
# bf16 storage helpers (bit manipulation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 -> bf16 (round to nearest, ties to even); return uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


class Bf16Tensor:
    """A tensor stored as bf16 bit patterns; indexing decodes to float32."""

    def __init__(self, bits: np.ndarray):
        assert bits.dtype == np.uint16
        self.bits = bits

    @classmethod
    def from_f32(cls, a: np.ndarray) -> "Bf16Tensor":
        return cls(f32_to_bf16_bits(a))

    @property
    def shape(self):
        return self.bits.shape

    def __len__(self):
        return self.bits.shape[0]

    def __getitem__(self, idx) -> np.ndarray:
        return bf16_bits_to_f32(self.bits[idx])

    def __array__(self, dtype=None, copy=None):
        a = bf16_bits_to_f32(self.bits)
        return a if dtype is None else a.astype(dtype)


def decode(t) -> np.ndarray:
    """float32 view of a stored tensor (Bf16Tensor or ndarray)."""
    return np.asarray(t, dtype=np.float32) if isinstance(t, Bf16Tensor) else np.asarray(t)


# ----------------------------------------------------------------------------
# configurations (the five benchmark layers)
# ----------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    N: int
    d: int
    f: int
    E: int
    k: int
    V: int
    dtype: int
    act: int
    backward: bool
    skew: str            # "none" | "log" | "zipf" | "dirichlet"
    skew_s: float = 0.0  # strength (multiplier of ln(1/rank), or Dirichlet alpha)
    max_rep: int = 1
    cfg_id: int = 0

    @property
    def A(self) -> int:
        return self.N * self.k


CONFIGS = {
    "tiny": LayerConfig("tiny", 256, 64, 256, 4, 1, 4, DT_F32, ACT_RELU, False, "none", cfg_id=1),
    "bert": LayerConfig("bert", 8192, 768, 3072, 16, 2, 18, DT_BF16, ACT_GELU_ERF, False,
                        "log", 2.0, max_rep=2, cfg_id=2),
    "gpt_m": LayerConfig("gpt_m", 16384, 1024, 4096, 32, 2, 48, DT_BF16, ACT_GELU_ERF, True,
                         "zipf", 1.2, max_rep=4, cfg_id=3),
    "swin": LayerConfig("swin", 32768, 512, 2048, 32, 1, 40, DT_BF16, ACT_GELU_ERF, True,
                        "dirichlet", 0.5, max_rep=8, cfg_id=4),
    "gpt_xl": LayerConfig("gpt_xl", 65536, 2048, 8192, 64, 2, 96, DT_BF16, ACT_GELU_ERF, True,
                          "zipf", 1.5, max_rep=8, cfg_id=5),
}
CONFIG_ORDER = ["tiny", "bert", "gpt_m", "swin", "gpt_xl"]


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some sizes replaced (reduced-size parity cases)."""
    return dataclasses.replace(cfg, **kw)


# ----------------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------------
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def _normal_f32(seed: int, stream: int, shape, std: float) -> np.ndarray:
    a = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def _store(a: np.ndarray, dtype: int):
    return Bf16Tensor.from_f32(a) if dtype == DT_BF16 else np.ascontiguousarray(a, dtype=np.float32)


def _expert_weights(seed: int, base_stream: int, E: int, rows: int, cols: int, dtype: int):
    """[E, rows, cols] ~ N(0, std 0.02), one independent stream per expert."""
    if dtype == DT_BF16:
        out = np.empty((E, rows, cols), dtype=np.uint16)
    else:
        out = np.empty((E, rows, cols), dtype=np.float32)

    def fill(e):
        a = _normal_f32(seed, base_stream + e, (rows, cols), 0.02)
        out[e] = f32_to_bf16_bits(a) if dtype == DT_BF16 else a

    if E * rows * cols > (1 << 24):
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(E)))
    else:
        for e in range(E):
            fill(e)
    return Bf16Tensor(out) if dtype == DT_BF16 else out


def target_shares(cfg: LayerConfig, seed: int, drift: int = 0):
    """Share of the N*k assignments that each expert should receive under the configured routing
    law (sums to 1), or None when the configuration states the logit bias itself ("log") or has no
    skew.  "zipf": share proportional to rank^-s, ranks dealt by a seeded permutation that rotates by
    four places per drift (the hot set moves smoothly); "dirichlet": one seeded draw of
    Dirichlet(alpha).  No expert can take more than 1/k of the assignments (k distinct experts per
    token): shares above that are cut to 1/k and the rest rescaled."""
    E, k = cfg.E, cfg.k
    if cfg.skew == "zipf":
        pi0 = _rng(seed, 7).permutation(E)
        rank = (pi0 + 4 * drift) % E
        p = (rank + 1.0) ** (-cfg.skew_s)
    elif cfg.skew == "dirichlet":
        p = np.maximum(_rng(seed, 7).dirichlet(np.full(E, cfg.skew_s)), 1e-7)
    else:
        return None
    p = p / p.sum()
    cap = 0.98 / k if k > 1 else 1.0
    for _ in range(E):
        over = p > cap
        if not over.any():
            break
        rest = 1.0 - cap * over.sum()
        p = np.where(over, cap, p * rest / p[~over].sum())
    return p


def _norm_cdf(z):
    from math import sqrt
    try:
        from scipy.special import ndtr
        return ndtr(z)
    except ImportError:            # pragma: no cover
        from math import erf
        return 0.5 * (1.0 + np.vectorize(erf)(z / sqrt(2.0)))


def inclusion_probabilities(b: np.ndarray, sigma: np.ndarray, k: int, grid: int = 481) -> np.ndarray:
    """P(expert e is among the k largest of l_j = b_j + sigma_j z_j, z iid N(0,1)), for every e.

    This is the statistics of the synthetic gate INPUTS, not the gate: with x ~ N(0, I) the
    logit noise of expert j is exactly N(0, |W_g[:, j]|^2), independent over tokens.  Quadrature
    over z_e; the number of rivals above l_e is Poisson-binomial, summed by a k-state recursion."""
    b = np.asarray(b, dtype=np.float64)
    sigma = np.asarray(sigma, dtype=np.float64)
    E = b.shape[0]
    u = np.linspace(-8.0, 8.0, grid)
    wq = np.exp(-0.5 * u * u)
    wq /= wq.sum()
    le = b[:, None] + sigma[:, None] * u[None, :]                    # [E, G]  value of l_e
    q = 1.0 - _norm_cdf((le[:, :, None] - b[None, None, :]) / sigma[None, None, :])   # [E, G, E]  P(l_j > l_e)
    idx = np.arange(E)
    q[idx, :, idx] = 0.0
    state = np.zeros((k, E, grid))                                    # state[c] = P(c rivals above so far)
    state[0] = 1.0
    for j in range(E):
        qj = q[:, :, j]
        for c in range(k - 1, 0, -1):
            state[c] = state[c] * (1.0 - qj) + state[c - 1] * qj
        state[0] = state[0] * (1.0 - qj)
    return (state.sum(axis=0) * wq[None, :]).sum(axis=1)


def solve_bias(p: np.ndarray, sigma: np.ndarray, k: int, tol: float = 2e-3, iters: int = 60) -> np.ndarray:
    """Logit biases b (max b = 0) under which `inclusion_probabilities` equals k*p: the expected
    share of assignments per expert is then p.  Secant iteration per coordinate.  (Layers with
    hundreds of experts, which only the edge-case tests use, get a coarser quadrature and
    tolerance: the evaluation costs E*E*k per quadrature point.)"""
    p = np.asarray(p, dtype=np.float64)
    grid = 481
    if p.shape[0] * k > 512:
        grid, tol, iters = 97, max(tol, 2e-2), min(iters, 25)
    _incl = inclusion_probabilities
    inclusion = lambda bb, ss, kk: _incl(bb, ss, kk, grid)          # noqa: E731
    want = np.log(np.minimum(k * p, 1.0 - 1e-9))
    b = np.log(p / p.max()) * np.mean(sigma)
    got = np.log(np.maximum(inclusion(b, sigma, k), 1e-300))
    slope = np.ones_like(b)
    for _ in range(iters):
        err = want - got
        if np.max(np.abs(err)) < tol:
            break
        step = np.clip(err / slope, -1.0, 1.0)
        b_new = b + step
        b_new -= b_new.max()
        got_new = np.log(np.maximum(inclusion(b_new, sigma, k), 1e-300))
        db = b_new - b
        ok = np.abs(db) > 1e-9
        est = np.where(ok, (got_new - got) / np.where(ok, db, 1.0), slope)
        slope = np.clip(np.where(np.isfinite(est) & (est > 0), est, slope), 0.2, 20.0)
        b, got = b_new, got_new
    return b


def expert_bias(cfg: LayerConfig, seed: int, drift: int = 0, sigma: np.ndarray | None = None) -> np.ndarray:
    """Per-expert additive logit bias b_e that produces the configured load skew.

    "log": the bias is stated outright, b_e = s * ln(1/(e+1)).  "zipf" / "dirichlet": the
    configuration states the routing law, so b is solved such that the expected share of
    assignments per expert equals `target_shares` given the logit noise the inputs carry
    (`sigma[e]` = standard deviation of expert e's logit noise; 1 when not given)."""
    E = cfg.E
    if cfg.skew == "none":
        return np.zeros(E, dtype=np.float64)
    if cfg.skew == "log":            # b_e = s * ln(1/(e+1)), hottest expert is e = 0
        return cfg.skew_s * np.log(1.0 / (np.arange(E) + 1.0))
    p = target_shares(cfg, seed, drift)
    if sigma is None:
        sigma = np.ones(E)
    return solve_bias(p, np.asarray(sigma, dtype=np.float64), cfg.k)


@dataclasses.dataclass
class LayerInputs:
    cfg: LayerConfig
    seed: int
    x: object        # [N, d]
    wg: object       # [d, E]
    w1: object       # [E, d, f]
    w2: object       # [E, f, d]
    dy: object       # [N, d] or None
    bias: np.ndarray  # [E] float64, the skew bias written into wg's last row


def make_gate_weights(cfg: LayerConfig, seed: int, drift: int = 0):
    """W_g [d,E] ~ N(0,1)/sqrt(d); for skewed configs the last row holds b_e.

    The bias is solved against the noise these very weights give the logits: features 0..d-2 of x
    are N(0,1), so expert e's logit noise has standard deviation |W_g[0:d-1, e]| (of the values as
    stored, i.e. after rounding to the config dtype)."""
    wg = _normal_f32(seed, 2, (cfg.d, cfg.E), 1.0 / math.sqrt(cfg.d))
    if cfg.skew == "none":
        return _store(wg, cfg.dtype), np.zeros(cfg.E)
    stored = decode(_store(wg[:cfg.d - 1], cfg.dtype)).astype(np.float64)
    sigma = np.sqrt((stored * stored).sum(axis=0))
    b = expert_bias(cfg, seed, drift, sigma)
    wg[cfg.d - 1, :] = b.astype(np.float32)
    return _store(wg, cfg.dtype), b


def make_layer_inputs(cfg: LayerConfig, seed: int | None = None, drift: int = 0,
                      with_weights: bool = True) -> LayerInputs:
    """Draw x, W_g, W1, W2 (and dY for training configs) for one layer.

    Skewed configs reserve the last input feature as a constant 1 so that the
    bias-free gate of the paper's Eq. 3 sees logits  x.W_g + b_e.
    """
    if seed is None:
        seed = BASE_SEED + cfg.cfg_id
    if cfg.skew == "none":
        x = _normal_f32(seed, 1, (cfg.N, cfg.d), 1.0 / math.sqrt(cfg.d))
    else:
        x = _normal_f32(seed, 1, (cfg.N, cfg.d), 1.0)
        x[:, cfg.d - 1] = 1.0
    wg, b = make_gate_weights(cfg, seed, drift)
    w1 = w2 = None
    if with_weights:
        w1 = _expert_weights(seed, 1000, cfg.E, cfg.d, cfg.f, cfg.dtype)
        w2 = _expert_weights(seed, 5000, cfg.E, cfg.f, cfg.d, cfg.dtype)
    dy = _store(_normal_f32(seed, 3, (cfg.N, cfg.d), 1.0), cfg.dtype) if cfg.backward else None
    return LayerInputs(cfg, seed, _store(x, cfg.dtype), wg, w1, w2, dy, b)


def sample_topk_idx(cfg: LayerConfig, seed: int, log_p: np.ndarray | None = None) -> np.ndarray:
    """Draw top-k expert ids directly (Gumbel top-k on ln p_e), bypassing the gate.

    Used for stage-level routing tests and benches that need an exact skew.
    Returns int32 [N, k] with k distinct experts per token.
    """
    if log_p is None:
        p = target_shares(cfg, seed)
        log_p = np.log(p) if p is not None else expert_bias(cfg, seed)
    g = _rng(seed, 11).gumbel(size=(cfg.N, cfg.E))
    s = g + np.asarray(log_p, dtype=np.float64)[None, :]
    return np.argsort(-s, axis=1, kind="stable")[:, :cfg.k].astype(np.int32)


# ----------------------------------------------------------------------------
# placement tables
# ----------------------------------------------------------------------------
def identity_placement(E: int):
    return np.arange(E + 1, dtype=np.int32), np.arange(E, dtype=np.int32)


def placement_from_loads(loads, V: int, max_rep: int, shuffle_seed: int | None = None):
    """Greedy stand-in for the paper's Policy Maker (Alg. 2's capacity rule).

    Every expert starts with one vExpert (slot v = e).  Each of the V-E spare
    slots E, E+1, ... goes to the expert with the largest load per replica
    I_e / n_e among experts with fewer than `max_rep` replicas (ties -> lowest
    e).  Returns CSR (rep_off[E+1], rep_ids[V]) int32; with `shuffle_seed` the
    slot ids are passed through a seeded permutation.
    """
    loads = np.asarray(loads, dtype=np.float64)
    E = loads.shape[0]
    assert V >= E
    reps = [[e] for e in range(E)]
    for slot in range(E, V):
        best, best_cap = -1, -1.0
        for e in range(E):
            if len(reps[e]) >= max_rep:
                continue
            cap = loads[e] / len(reps[e])
            if cap > best_cap:
                best, best_cap = e, cap
        if best < 0:
            raise ValueError("V exceeds E * max_rep")
        reps[best].append(slot)
    rep_off = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        rep_off[e + 1] = rep_off[e] + len(reps[e])
    rep_ids = np.array([v for r in reps for v in r], dtype=np.int32)
    if shuffle_seed is not None:
        perm = _rng(shuffle_seed, 13).permutation(V).astype(np.int32)
        rep_ids = perm[rep_ids]
    return rep_off, rep_ids


def prior_loads(cfg: LayerConfig, seed: int | None = None, drift: int = 0) -> np.ndarray:
    """Expected loads before any step has been observed: N*k*target share; where the configuration
    states the bias instead of the law, N*k*softmax(b) capped at N per expert."""
    if seed is None:
        seed = BASE_SEED + cfg.cfg_id
    p = target_shares(cfg, seed, drift)
    if p is None:
        b = expert_bias(cfg, seed, drift)
        p = np.exp(b - b.max())
        p /= p.sum()
    return np.minimum(cfg.A * p, cfg.N)


def config_placement(cfg: LayerConfig, loads=None, seed: int | None = None, drift: int = 0,
                     shuffle_seed: int | None = None):
    """The placement table of a benchmark configuration."""
    if cfg.V == cfg.E:
        return identity_placement(cfg.E)
    if cfg.name == "bert" and loads is None:
        # the two hottest experts (0 and 1 under b_e = 2 ln 1/(e+1)) get a second replica
        rep_off = np.zeros(cfg.E + 1, dtype=np.int32)
        ids = []
        for e in range(cfg.E):
            r = [e] + ([cfg.E + e] if e < 2 else [])
            ids += r
            rep_off[e + 1] = rep_off[e] + len(r)
        return rep_off, np.array(ids, dtype=np.int32)
    if loads is None:
        loads = prior_loads(cfg, seed, drift)
    return placement_from_loads(loads, cfg.V, cfg.max_rep, shuffle_seed)
