"""Seeded synthetic workloads for the SLO-NN hot path.

This module only *generates data*: weights, biases, query/build inputs, the
hash-node id lists and the keep fractions.  It holds none of the method's
arithmetic (no dot products, no hashing, no selection) so that the CPU oracle
and the HIP path can both be fed from it without sharing any computation.

Every number comes from one counter-based generator (splitmix64 finaliser over
``seed``, ``stream`` and an element counter), so any element can be recomputed
in isolation and arrays are reproducible regardless of how they are chunked.

The paper's datasets and trained models (Table 1) are not available; the shapes
below stand in for them: a FMNIST-like 784-112-10 net, two scaled-up ReLU MLPs,
a wide sparse-input extreme-classification net with the Node Activator at the
output layer only (Section 4, "Model Pruning"), and a deep bf16 MLP with mixed
per-query keep fractions.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_U64 = np.uint64
_MASK53 = (1 << 53) - 1


# --------------------------------------------------------------------------- #
# counter-based random numbers
# --------------------------------------------------------------------------- #
def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function, vectorised over a uint64 array."""
    z = z.copy()
    z ^= z >> _U64(30)
    z *= _U64(0xBF58476D1CE4E5B9)
    z ^= z >> _U64(27)
    z *= _U64(0x94D049BB133111EB)
    z ^= z >> _U64(31)
    return z


def random_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """``count`` 64-bit words for counters ``start .. start+count-1``."""
    with np.errstate(over="ignore"):
        base = _mix64(np.array([(seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03
                                 + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF], dtype=_U64))[0]
        ctr = np.arange(start, start + count, dtype=_U64)
        return _mix64(base + (ctr + _U64(1)) * _U64(0x9E3779B97F4A7C15))


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniform in [0, 1) with 53 random bits."""
    return (random_u64(seed, stream, start, count) >> _U64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 standard normals (Box-Muller, one normal per counter)."""
    u1 = uniform01(seed, 2 * stream, start, count)
    u2 = uniform01(seed, 2 * stream + 1, start, count)
    r = np.sqrt(-2.0 * np.log1p(-u1))          # 1-u1 in (0, 1]
    return r * np.cos(2.0 * np.pi * u2)


def _chunks(total: int, step: int = 1 << 22):
    for s in range(0, total, step):
        yield s, min(step, total - s)


def _fill(fn, seed: int, stream: int, total: int, dtype) -> np.ndarray:
    out = np.empty(total, dtype=dtype)
    for s, c in _chunks(total):
        out[s:s + c] = fn(seed, stream, s, c)
    return out


# --------------------------------------------------------------------------- #
# bf16 storage (round-to-nearest-even on the fp32 bit pattern)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# model and inputs
# --------------------------------------------------------------------------- #
W_F32 = 0
W_BF16 = 1
ACT_NONE = 0
ACT_RELU = 1
ACT_SOFTMAX = 2


@dataclass
class LayerData:
    d_in: int
    d_out: int
    act: int
    w_dtype: int
    W: np.ndarray                 # [d_out][d_in] float32, or uint16 bf16 bit patterns
    bias: np.ndarray              # [d_out] float32
    K: int = 0
    L: int = 0
    list_cap: int = 0
    hash_nodes: Optional[np.ndarray] = None     # int32 [L*K], table-major


def make_mlp(dims: Sequence[int], seed: int = 0, w_dtype: int = W_F32,
             last_act: int = ACT_NONE) -> List[LayerData]:
    """He-normal weights N(0, 2/fan_in) and small biases 0.01*N(0,1)."""
    layers = []
    for l in range(len(dims) - 1):
        d, n = int(dims[l]), int(dims[l + 1])
        w = _fill(normal01, seed, 10 + 2 * l, n * d, np.float64) * np.sqrt(2.0 / d)
        b = _fill(normal01, seed, 11 + 2 * l, n, np.float64) * 0.01
        w32 = w.astype(np.float32).reshape(n, d)
        W = f32_to_bf16_bits(w32).reshape(n, d) if w_dtype == W_BF16 else w32
        act = ACT_RELU if l < len(dims) - 2 else last_act
        layers.append(LayerData(d, n, act, w_dtype, W, b.astype(np.float32)))
    return layers


def inputs_uniform_half_zero(N: int, d: int, seed: int) -> np.ndarray:
    """Each element is exactly 0 with probability 1/2, else uniform in [0, 1)."""
    vals = _fill(uniform01, seed, 1, N * d, np.float64)
    gate = _fill(uniform01, seed, 2, N * d, np.float64)
    return np.where(gate < 0.5, 0.0, vals).astype(np.float32).reshape(N, d)


def inputs_normal_clipped(N: int, d: int, seed: int, clip: Optional[float] = 3.0) -> np.ndarray:
    x = _fill(normal01, seed, 3, N * d, np.float64)
    if clip is not None:
        x = np.clip(x, -clip, clip)
    return x.astype(np.float32).reshape(N, d)


def inputs_ell(N: int, d: int, nnz: int, seed: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Sparse inputs: ``nnz`` distinct uniform column indices per row, values U[0,1).

    Returns (idx int32 [N][nnz], val float32 [N][nnz], cnt int32 [N]).  Distinct
    indices are obtained by redrawing duplicates with fresh counters.
    """
    idx = np.empty((N, nnz), dtype=np.int32)
    draws = (random_u64(seed, 4, 0, N * nnz) % _U64(d)).astype(np.int64).reshape(N, nnz)
    extra = N * nnz
    for r in range(N):
        row = draws[r]
        while True:
            _, first = np.unique(row, return_index=True)
            if len(first) == nnz:
                break
            dup = np.setdiff1d(np.arange(nnz), first)
            row[dup] = (random_u64(seed, 4, extra, len(dup)) % _U64(d)).astype(np.int64)
            extra += len(dup)
        idx[r] = row
    val = _fill(uniform01, seed, 5, N * nnz, np.float64).astype(np.float32).reshape(N, nnz)
    return idx, val, np.full(N, nnz, dtype=np.int32)


def keep_uniform(N: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """Per-query keep fractions uniform in [lo, hi] (mixed SLOs in one batch)."""
    return (lo + (hi - lo) * uniform01(seed, 6, 0, N)).astype(np.float32)


def hash_node_draws(K: int, L: int, seed: int) -> np.ndarray:
    """The K*L uniform draws in [0, 1) that the sampling of a layer's hash nodes consumes
    (an input to both implementations of that sampling)."""
    return uniform01(seed, 7, 0, K * L)


# --------------------------------------------------------------------------- #
# the benchmark configurations
# --------------------------------------------------------------------------- #
@dataclass
class Config:
    name: str
    dims: Tuple[int, ...]
    w_dtype: int
    last_act: int
    n_inputs: int
    input_kind: str                       # "u01_half_zero" | "normal_clip3" | "normal" | "ell"
    hashed_layers: Tuple[int, ...]        # indices of layers carrying a Node Activator
    K: int
    L: int
    keeps: Tuple[float, ...]
    batches: Tuple[int, ...]
    ell_nnz: int = 0
    keep_range: Optional[Tuple[float, float]] = None
    note: str = ""


CONFIGS = {
    "C1": Config("C1", (784, 112, 10), W_F32, ACT_SOFTMAX, 1000, "u01_half_zero",
                 (0,), 6, 10, (0.25,), (1, 64), note="FMNIST-shaped, latency-bound"),
    "C2": Config("C2", (784, 1024, 1024, 10), W_F32, ACT_NONE, 10000, "u01_half_zero",
                 (0, 1), 8, 16, (0.05, 0.1, 0.25, 0.5, 1.0), (256,)),
    "C3": Config("C3", (3072, 4096, 4096, 4096, 100), W_F32, ACT_NONE, 50000, "normal_clip3",
                 (0, 1, 2), 10, 32, (0.05, 0.1, 0.25, 0.5), (1, 32, 1024)),
    "C4": Config("C4", (100000, 128, 100000), W_F32, ACT_SOFTMAX, 12800, "ell",
                 (1,), 12, 50, (0.005,), (128,), ell_nnz=100),
    "C5": Config("C5", (1024,) + (8192,) * 6 + (1000,), W_BF16, ACT_NONE, 20000, "normal",
                 (0, 1, 2, 3, 4, 5), 12, 64, (), (2048,), keep_range=(0.02, 0.3)),
}


def inputs_clustered(N: int, d: int, seed: int, n_clusters: int, spread: float = 0.3,
                     clip: Optional[float] = 3.0) -> np.ndarray:
    """Inputs with class structure (not one of the benchmark configurations; for the study of
    batches ordered by LSH key): ``n_clusters`` centres drawn N(0,1) once (seed-independent
    stream), each input = its centre + ``spread`` * N(0,1), the centre picked uniformly at random
    per input, arrival order random."""
    centres = _fill(normal01, 12345, 8, n_clusters * d, np.float64).reshape(n_clusters, d)
    which = (random_u64(seed, 9, 0, N) % _U64(n_clusters)).astype(np.int64)
    x = centres[which] + spread * _fill(normal01, seed, 3, N * d, np.float64).reshape(N, d)
    if clip is not None:
        x = np.clip(x, -clip, clip)
    return x.astype(np.float32)


def make_inputs(cfg: Config, N: int, seed: int):
    d = cfg.dims[0]
    if cfg.input_kind == "u01_half_zero":
        return inputs_uniform_half_zero(N, d, seed)
    if cfg.input_kind == "normal_clip3":
        return inputs_normal_clipped(N, d, seed, 3.0)
    if cfg.input_kind == "normal":
        return inputs_normal_clipped(N, d, seed, None)
    if cfg.input_kind == "ell":
        return inputs_ell(N, d, cfg.ell_nnz, seed)
    raise ValueError(cfg.input_kind)
