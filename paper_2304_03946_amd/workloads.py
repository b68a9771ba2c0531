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


def expert_bias(cfg: LayerConfig, seed: int, drift: int = 0) -> np.ndarray:
    """Per-expert additive logit bias b_e that produces the configured load skew."""
    E = cfg.E
    if cfg.skew == "none":
        return np.zeros(E, dtype=np.float64)
    if cfg.skew == "log":            # b_e = s * ln(1/(e+1)), hottest expert is e = 0
        return cfg.skew_s * np.log(1.0 / (np.arange(E) + 1.0))
    if cfg.skew == "zipf":           # Zipf ranks through a seeded permutation, rotated by drift
        pi0 = _rng(seed, 7).permutation(E)
        rank = (pi0 + 4 * drift) % E
        return cfg.skew_s * np.log(1.0 / (rank + 1.0))
    if cfg.skew == "dirichlet":
        p = _rng(seed, 7).dirichlet(np.full(E, cfg.skew_s))
        return np.maximum(np.log(np.maximum(p, 1e-300)), -20.0)
    raise ValueError(cfg.skew)


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
    """W_g [d,E] ~ N(0,1)/sqrt(d); for skewed configs the last row holds b_e."""
    wg = _normal_f32(seed, 2, (cfg.d, cfg.E), 1.0 / math.sqrt(cfg.d))
    b = expert_bias(cfg, seed, drift)
    if cfg.skew != "none":
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
        log_p = expert_bias(cfg, seed)
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
    """Loads implied by the skew bias alone: N*k*softmax(b), capped at N per expert."""
    if seed is None:
        seed = BASE_SEED + cfg.cfg_id
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
