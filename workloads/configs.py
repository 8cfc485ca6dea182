"""Seeded generators for the five benchmark configurations.

Every generator is a pure function of (config id, variant): numpy's
``default_rng(SEED_BASE + 10*config + variant)`` drives all draws.  Matrices are
int8, row-major ``rows x cols``; the vector multiplies from the left, so an
activation has ``rows`` entries and the product has ``cols`` entries.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

SEED_BASE = 2411063600


def seed_for(config: int, variant: int = 0) -> int:
    return SEED_BASE + 10 * int(config) + int(variant)


def binary_matrix(rng: np.random.Generator, rows: int, cols: int, p_one: float = 0.5) -> np.ndarray:
    """Entries i.i.d. Bernoulli(p_one) in {0,1}; drawn in row chunks to bound memory."""
    A = np.empty((rows, cols), dtype=np.int8)
    step = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        u = rng.random((r1 - r0, cols), dtype=np.float32)
        A[r0:r1] = (u < np.float32(p_one)).astype(np.int8)
    return A


def _ternary_from_uniform(u: np.ndarray, p_zero: float) -> np.ndarray:
    """Map uniforms in [0,1) to {-1,0,1} with P(0)=p_zero and P(+1)=P(-1)=(1-p_zero)/2."""
    p_side = np.float32((1.0 - p_zero) / 2.0)
    out = np.zeros(u.shape, dtype=np.int8)
    out[u < p_side] = 1
    out[u >= np.float32(1.0) - p_side] = -1
    return out


def ternary_matrix(rng: np.random.Generator, rows: int, cols: int, p_zero: float = 1.0 / 3.0) -> np.ndarray:
    """Entries i.i.d. over {-1,0,1} with P(0)=p_zero and the rest split evenly."""
    A = np.empty((rows, cols), dtype=np.int8)
    step = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        u = rng.random((r1 - r0, cols), dtype=np.float32)
        A[r0:r1] = _ternary_from_uniform(u, p_zero)
    return A


def correlated_ternary_matrix(
    rng: np.random.Generator,
    rows: int,
    cols: int,
    p_zero: float = 0.6,
    n_prototypes: int = 64,
    p_resample: float = 0.05,
) -> np.ndarray:
    """Rows correlated through a small set of prototype rows (skewed segment sizes).

    ``n_prototypes`` rows are drawn i.i.d. from the ternary law; every matrix row
    copies one prototype chosen uniformly at random, then each of its entries is
    independently redrawn from the same law with probability ``p_resample``.
    """
    protos = _ternary_from_uniform(rng.random((n_prototypes, cols), dtype=np.float32), p_zero)
    which = rng.integers(0, n_prototypes, size=rows)
    A = np.empty((rows, cols), dtype=np.int8)
    step = max(1, (1 << 23) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        chunk = protos[which[r0:r1]]
        redo = rng.random((r1 - r0, cols), dtype=np.float32) < np.float32(p_resample)
        fresh = _ternary_from_uniform(rng.random((r1 - r0, cols), dtype=np.float32), p_zero)
        A[r0:r1] = np.where(redo, fresh, chunk)
    return A


def make_activations(rng: np.random.Generator, batch: int, rows: int, dtype: str) -> np.ndarray:
    """``batch x rows`` activations: fp32 i.i.d. N(0,1), or int8 uniform on [-127,127]."""
    if dtype == "f32":
        return rng.standard_normal((batch, rows), dtype=np.float32)
    if dtype == "i8":
        return rng.integers(-127, 128, size=(batch, rows), dtype=np.int8)
    raise ValueError(f"unknown activation dtype {dtype!r}")


@dataclass(frozen=True)
class Workload:
    """One named matrix of a configuration, generated on demand."""

    name: str
    config: int
    variant: int
    kind: str  # "binary" | "ternary" | "ternary_correlated"
    rows: int
    cols: int
    k: int
    p_zero: float = 0.0
    batches: Tuple[int, ...] = (1,)
    dtypes: Tuple[str, ...] = ("f32",)
    extra: Dict[str, float] = field(default_factory=dict)

    @property
    def seed(self) -> int:
        return seed_for(self.config, self.variant)

    def matrix(self) -> np.ndarray:
        rng = np.random.default_rng(self.seed)
        if self.kind == "binary":
            return binary_matrix(rng, self.rows, self.cols, 0.5)
        if self.kind == "ternary":
            return ternary_matrix(rng, self.rows, self.cols, self.p_zero)
        if self.kind == "ternary_correlated":
            return correlated_ternary_matrix(rng, self.rows, self.cols, self.p_zero, 64, 0.05)
        raise ValueError(self.kind)

    def activations(self, batch: int, dtype: str) -> np.ndarray:
        # an independent stream, so that v does not depend on how A consumed its draws
        rng = np.random.default_rng([self.seed, 1, batch, 0 if dtype == "f32" else 1])
        return make_activations(rng, batch, self.rows, dtype)


def _llm_block() -> List[Workload]:
    """Config 4: seven ternary matrices shaped like one ~2B-parameter 1.58-bit transformer block."""
    shapes = [
        ("attn_q", 2560, 2560),
        ("attn_k", 2560, 2560),
        ("attn_v", 2560, 2560),
        ("attn_o", 2560, 2560),
        ("mlp_gate", 2560, 6912),
        ("mlp_up", 2560, 6912),
        ("mlp_down", 6912, 2560),
    ]
    return [
        Workload(f"llm_block.{n}", 4, i, "ternary", r, c, 10, p_zero=0.5, batches=(1, 16), dtypes=("f32",))
        for i, (n, r, c) in enumerate(shapes)
    ]


CONFIGS: Dict[int, List[Workload]] = {
    1: [Workload("binary_1k", 1, 0, "binary", 1024, 1024, 8, batches=(1,), dtypes=("i8",))],
    2: [Workload("ternary_4k", 2, 0, "ternary", 4096, 4096, 10, p_zero=1.0 / 3.0, batches=(1,), dtypes=("f32",))],
    3: [Workload("binary_16k", 3, 0, "binary", 16384, 16384, 12, batches=(1, 8), dtypes=("f32", "i8"))],
    4: _llm_block(),
    5: [
        Workload(
            "ternary_32k_correlated", 5, 0, "ternary_correlated", 32768, 32768, 13, p_zero=0.6,
            batches=(4,), dtypes=("f32",),
        )
    ],
}


def llm_block_stages() -> List[Tuple[str, List[Workload]]]:
    """Config 4 as the four matrix stages of one decode step of the block: the projections that read the
    same activation are one matrix (their columns side by side), so a stage is one index and one product.
    Returns (stage name, the config-4 matrices it concatenates) in the order the block applies them."""
    by = {w.name.split(".")[1]: w for w in CONFIGS[4]}
    return [
        ("qkv", [by["attn_q"], by["attn_k"], by["attn_v"]]),      # 2560 x 7680
        ("attn_o", [by["attn_o"]]),                               # 2560 x 2560
        ("gate_up", [by["mlp_gate"], by["mlp_up"]]),              # 2560 x 13824
        ("mlp_down", [by["mlp_down"]]),                           # 6912 x 2560
    ]


def stage_matrix(members: List[Workload]) -> np.ndarray:
    return np.ascontiguousarray(np.concatenate([w.matrix() for w in members], axis=1))


def get(name: str) -> Workload:
    for ws in CONFIGS.values():
        for w in ws:
            if w.name == name:
                return w
    raise KeyError(name)
