"""Seeded synthetic inputs for the five DiT-linear workloads.

This module only draws random tensors; it contains none of the method's
arithmetic (no norms, thresholds, scales or rounding) and is the single piece
shared by the oracle-side and GPU-side tests and by ``bench.py``.  Tensors are
made once on the host with ``numpy.random.default_rng(seed)`` as fp32 and
handed unchanged to both sides.

The paper's real workloads are the weights and activations of a Wan-1.3B-style
DiT (30 blocks x 10 linears, hidden 1536, FFN 8960) run chunk by chunk
(3 latent frames = 3*30*52 = 4680 tokens per call); neither weights nor
prompts are available, so only the shapes and the outlier structure (a few
percent of input channels with a much larger norm, heterogeneous over layer
type and depth, ffn-down prominent, cross-attn v smooth) are reproduced.

  seed(config, ordinal) = 260521072 + 1000*config + ordinal
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 260521072
HIDDEN, FFN = 1536, 8960          # Wan-1.3B-style DiT
HIDDEN_L, FFN_L = 5120, 13824     # 14B-scale DiT
M_CHUNK = 4680                    # 3 latent frames x 30 x 52 tokens
M_FRAME = 1560
M_THIRD = 520
M_TEXT = 512
N_BLOCKS = 30


@dataclass
class LayerSpec:
    config: int
    ordinal: int
    name: str
    M: int
    K: int
    N: int
    n_outlier: int                         # planted outlier input channels
    w_std: float = 0.02
    w_mult: Tuple[float, float] = (10.0, 40.0)   # per-column multiplier ~ U[lo, hi]
    x_mult: float = 15.0
    fixed_channels: Optional[Tuple[int, ...]] = None   # activation channels if given explicitly
    bias_std: float = 0.01
    tags: dict = field(default_factory=dict)

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.config + self.ordinal

    @property
    def macs(self) -> int:
        return self.M * self.K * self.N


def make_weight(spec: LayerSpec):
    """W f32[N,K], bias f32[N], planted weight columns (sorted int64[c])."""
    rng = np.random.default_rng(spec.seed)
    W = rng.standard_normal((spec.N, spec.K), dtype=np.float32)
    W *= np.float32(spec.w_std)
    cols = np.sort(rng.choice(spec.K, spec.n_outlier, replace=False)) if spec.n_outlier else \
        np.zeros(0, np.int64)
    lo, hi = spec.w_mult
    mult = rng.uniform(lo, hi, size=cols.shape[0]).astype(np.float32)
    for c, m in zip(cols, mult):
        W[:, c] *= m
    bias = (rng.standard_normal(spec.N, dtype=np.float32) * np.float32(spec.bias_std))
    return W, bias, cols


def make_activation(spec: LayerSpec, cols=None, rows: Optional[int] = None):
    """X f32[M,K] ~ N(0,1) with the outlier channels scaled by ``x_mult``.

    ``rows`` draws only the first ``rows`` tokens (same values as the full draw's
    first rows are NOT guaranteed; a reduced draw is its own seeded tensor).
    """
    M = spec.M if rows is None else rows
    rng = np.random.default_rng(spec.seed + 500)
    X = rng.standard_normal((M, spec.K), dtype=np.float32)
    if spec.fixed_channels is not None:
        ch = np.asarray(spec.fixed_channels, dtype=np.int64)
    else:
        ch = np.asarray(cols if cols is not None else [], dtype=np.int64)
    if ch.size:
        X[:, ch] *= np.float32(spec.x_mult)
    return X


def make_layer(spec: LayerSpec, rows: Optional[int] = None):
    W, bias, cols = make_weight(spec)
    X = make_activation(spec, cols, rows)
    return dict(X=X, W=W, bias=bias, planted=cols, spec=spec)


# ------------------------------------------------------------------ configs

def config1() -> List[LayerSpec]:
    return [LayerSpec(1, 0, "cfg1.linear", 256, HIDDEN, HIDDEN, 8, 0.02, (25.0, 25.0), 20.0,
                      fixed_channels=tuple(range(96, HIDDEN, 192)))]


def config2() -> List[LayerSpec]:
    out, o = [], 0
    shapes = [("q", HIDDEN, HIDDEN), ("k", HIDDEN, HIDDEN), ("v", HIDDEN, HIDDEN),
              ("o", HIDDEN, HIDDEN), ("ffn_up", HIDDEN, FFN), ("ffn_down", FFN, HIDDEN)]
    for name, K, N in shapes:
        for c in (0, 4, 16, 64):
            out.append(LayerSpec(2, o, "cfg2.%s.c%d" % (name, c), M_CHUNK, K, N, c))
            o += 1
    return out


_CFG3_TYPES = [  # (name, M, K, N, hi)
    ("self_q", M_CHUNK, HIDDEN, HIDDEN, 32), ("self_k", M_CHUNK, HIDDEN, HIDDEN, 32),
    ("self_v", M_CHUNK, HIDDEN, HIDDEN, 32), ("self_o", M_CHUNK, HIDDEN, HIDDEN, 64),
    ("cross_q", M_CHUNK, HIDDEN, HIDDEN, 32), ("cross_k", M_TEXT, HIDDEN, HIDDEN, 16),
    ("cross_v", M_TEXT, HIDDEN, HIDDEN, 0), ("cross_o", M_CHUNK, HIDDEN, HIDDEN, 32),
    ("ffn_up", M_CHUNK, HIDDEN, FFN, 64), ("ffn_down", M_CHUNK, FFN, HIDDEN, 96),
]


def config3(blocks=range(N_BLOCKS)) -> List[LayerSpec]:
    out = []
    for d in blocks:
        depth = 0.5 + 0.5 * d / (N_BLOCKS - 1)
        for t, (name, M, K, N, hi) in enumerate(_CFG3_TYPES):
            o = d * len(_CFG3_TYPES) + t
            rng = np.random.default_rng(BASE_SEED + 3000 + o + 100000)
            c = int(rng.integers(0, int(round(hi * depth)) + 1))
            out.append(LayerSpec(3, o, "cfg3.b%02d.%s" % (d, name), M, K, N, c,
                                 tags=dict(block=d, type=name)))
    return out


def config4() -> List[LayerSpec]:
    out, o = [], 0
    for M in (M_FRAME, M_THIRD):
        for name, K, N in (("attn", HIDDEN, HIDDEN), ("ffn_up", HIDDEN, FFN),
                           ("ffn_down", FFN, HIDDEN)):
            for c in (0, 32):
                out.append(LayerSpec(4, o, "cfg4.M%d.%s.c%d" % (M, name, c), M, K, N, c))
                o += 1
    return out


def config5() -> List[LayerSpec]:
    out, o = [], 0
    for name, K, N in (("q", HIDDEN_L, HIDDEN_L), ("k", HIDDEN_L, HIDDEN_L),
                       ("v", HIDDEN_L, HIDDEN_L), ("o", HIDDEN_L, HIDDEN_L),
                       ("ffn_up", HIDDEN_L, FFN_L), ("ffn_down", FFN_L, HIDDEN_L)):
        for c in (0, 32, 128):
            out.append(LayerSpec(5, o, "cfg5.%s.c%d" % (name, c), M_CHUNK, K, N, c, 0.01,
                                 (30.0, 30.0), 20.0))
            o += 1
    return out


def config_layers(cfg: int) -> List[LayerSpec]:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[cfg]()


_BY_NAME = {}


def find_layer(name: str) -> LayerSpec:
    if not _BY_NAME:
        for cfg in (1, 2, 3, 4, 5):
            for s in config_layers(cfg):
                _BY_NAME[s.name] = s
    return _BY_NAME[name]


# The shape the benchmark spec quotes its target on: M=4680, 1536 -> 8960 with planted outliers.
TARGET_LAYER = "cfg2.ffn_up.c16"


def small_random_case(seed: int, M: int, N: int, K: int, n_outlier: int, w_std=0.02,
                      mult=(10.0, 40.0), x_mult=15.0):
    """Free-form seeded case for the tile/tail sweeps of the parity tests."""
    spec = LayerSpec(0, seed, "rand.%d" % seed, M, K, N, n_outlier, w_std, mult, x_mult)
    return make_layer(spec)
