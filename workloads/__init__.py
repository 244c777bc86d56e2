"""Seeded synthetic inputs for the ROBE-Z lookup path.

This module only produces INPUTS (array contents, token ids, bag boundaries,
upstream gradients) with the shapes and value distributions of the paper's
CriteoTB workload (Section 5.2: 26 categorical features, heavily skewed token
frequencies, one shared 100 MB array) and of the named benchmark
configurations.  It holds none of the method's arithmetic: no hashing, no
gather, no scatter.  Both the GPU tests/benchmark and the CPU oracle take
their inputs from here so that the two sides see identical bits.

Everything is NumPy on the host; callers upload what they need.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from functools import lru_cache
from typing import Optional, Tuple

import numpy as np

N_FEATURES = 26  # CriteoTB / Criteo Kaggle categorical feature count (Section 5.2)


@dataclass(frozen=True)
class Workload:
    name: str
    m: int                    # array length in floats
    d: int                    # embedding dimension
    Z: int                    # block size
    batch: int
    n_features: int
    cardinalities: Tuple[int, ...]
    id_dist: str              # "uniform" | "zipf"
    zipf_alpha: float
    use_sign: int
    bag_mean: Optional[float]  # None: single-hot; else Poisson mean of the bag size
    phases: str               # "fwd" | "fwd+bwd" | "fwd+bwd+adagrad" | "fwd+bwd+sgd"
    lr: float = 0.01
    eps: float = 1e-8
    hash_seed: int = 2108_02191
    dims: Optional[Tuple[int, ...]] = None   # per-table dimensions (tables of mixed dimensions); None: all d
    array_dtype: str = "f32"                 # "bf16": the array is quantised to bfloat16 for the forward pass

    @property
    def rows(self) -> int:
        return self.batch * self.n_features

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def log_spaced_cardinalities(lo: float = 10.0, hi: float = 4e7, n: int = N_FEATURES) -> Tuple[int, ...]:
    """n table sizes spaced geometrically from lo to hi (stand-in for CriteoTB's skewed table sizes)."""
    return tuple(int(round(lo * (hi / lo) ** (f / (n - 1)))) for f in range(n))


# Table sizes of the Criteo Kaggle dataset as the paper prints them (Appendix, "Criteo Kaggle
# Experiment": 26 categorical features, about 33 M values in total).
KAGGLE_CARDINALITIES = (1460, 583, 10131227, 2202608, 305, 24, 12517, 633, 3, 93145, 5683, 8351593,
                        3194, 27, 14992, 5461306, 10, 5652, 2173, 4, 7046547, 18, 15, 286181, 105, 142572)


def get(name: str) -> Workload:
    ls = log_spaced_cardinalities()
    if name == "tiny":
        return Workload("tiny", 2**20, 16, 4, 256, N_FEATURES, (1000,) * N_FEATURES, "uniform", 0.0, 0, None, "fwd+bwd")
    if name == "inference":
        return Workload("inference", 25_000_000, 128, 32, 32768, N_FEATURES, ls, "zipf", 1.05, 1, None, "fwd")
    if name == "training":
        return Workload("training", 25_000_000, 128, 32, 65536, N_FEATURES, ls, "zipf", 1.05, 0, None, "fwd+bwd+adagrad")
    if name.startswith("sweep_z"):
        Z = int(name[len("sweep_z"):])
        return Workload(name, 25_000_000, 128, Z, 32768, N_FEATURES, ls, "zipf", 1.05, 0, None, "fwd+bwd")
    if name.startswith("kaggle_z"):
        # the paper's second setting (Section 5.3): d = 16, 540 K parameters (1000x compression of
        # 540 M), Z in {1,2,4,8,16}, batch 2048, SGD for DLRM; ids synthetic (bounded Zipf per table)
        Z = int(name[len("kaggle_z"):])
        return Workload(name, 540_000, 16, Z, 2048, N_FEATURES, KAGGLE_CARDINALITIES, "zipf", 1.05, 0, None,
                        "fwd+bwd+sgd", lr=1.0)
    if name == "inference_bf16":
        # the inference configuration on a bfloat16 copy of the array (Section 2: quantisation composes
        # with the method; the paper measures no such configuration)
        return get("inference").scaled(name="inference_bf16", array_dtype="bf16")
    if name == "multihot_fwd_bf16":
        return get("multihot").scaled(name="multihot_fwd_bf16", phases="fwd", array_dtype="bf16")
    if name == "mixed_dims":
        # Tables of different dimensions in one array (Section 3.2, "Multiple embedding tables").  The
        # paper runs no such configuration; this one keeps the inference shapes and gives the small
        # tables small dimensions: 16 / 32 / 64 / 128 for the four quarters of the log-spaced sizes.
        dims = tuple(16 if f < 6 else 32 if f < 12 else 64 if f < 19 else 128 for f in range(N_FEATURES))
        return Workload("mixed_dims", 25_000_000, 128, 16, 32768, N_FEATURES, ls, "zipf", 1.05, 0, None, "fwd+bwd",
                        dims=dims)
    if name == "multihot":
        return Workload("multihot", 250_000_000, 128, 32, 16384, N_FEATURES, (40_000_000,) * N_FEATURES,
                        "zipf", 1.05, 0, 20.0, "fwd+bwd+adagrad")
    raise KeyError(name)


ALL = ("tiny", "inference", "training", "sweep_z1", "sweep_z8", "sweep_z32", "sweep_z128", "multihot",
       "kaggle_z1", "kaggle_z2", "kaggle_z4", "kaggle_z8", "kaggle_z16", "mixed_dims",
       "inference_bf16", "multihot_fwd_bf16")


def make_array(m: int, seed: int = 0) -> np.ndarray:
    """float32[m] ~ normal(0, 0.01)."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(m, dtype=np.float32)
    a *= np.float32(0.01)
    return a


@lru_cache(maxsize=2)
def _zipf_prefix(n_max: int, alpha: float) -> np.ndarray:
    w = np.arange(1, n_max + 1, dtype=np.float64)
    np.power(w, -alpha, out=w)
    np.cumsum(w, out=w)
    return w


def bounded_zipf(rng: np.random.Generator, n: int, cardinality: int, alpha: float,
                 prefix: Optional[np.ndarray] = None) -> np.ndarray:
    """n draws with Pr[id = r-1] proportional to r^-alpha, r = 1..cardinality (inverse CDF on the finite support)."""
    if prefix is None:
        prefix = _zipf_prefix(cardinality, alpha)
    u = rng.random(n) * prefix[cardinality - 1]
    r = np.searchsorted(prefix[:cardinality], u, side="right")
    np.minimum(r, cardinality - 1, out=r)
    return r.astype(np.int64)


def make_bag_sizes(w: Workload, seed: int) -> Optional[np.ndarray]:
    if w.bag_mean is None:
        return None
    rng = np.random.default_rng(seed + 7919)
    return rng.poisson(w.bag_mean, size=w.rows).astype(np.int64)


def make_indices(w: Workload, seed: int = 1) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Token ids and, for bag workloads, CSR offsets.

    single-hot: ids int64[batch, F].  bags: ids int64[nnz] in (b, f) bag order,
    offsets int64[batch*F + 1].  Feature f draws from its own generator
    (seed + f) over its own cardinality.
    """
    B, F = w.batch, w.n_features
    sizes = make_bag_sizes(w, seed)
    if sizes is None:
        per_row = np.ones(w.rows, dtype=np.int64)
    else:
        per_row = sizes
    offsets = np.zeros(w.rows + 1, dtype=np.int64)
    np.cumsum(per_row, out=offsets[1:])
    nnz = int(offsets[-1])
    ids = np.empty(nnz, dtype=np.int64)
    prefix = None
    if w.id_dist == "zipf":
        prefix = _zipf_prefix(max(w.cardinalities), w.zipf_alpha)
    # position of every token, grouped by the feature of its bag
    counts = per_row.reshape(B, F)
    starts = offsets[:-1].reshape(B, F)
    for f in range(F):
        rng = np.random.default_rng(seed * 1000 + f)
        n_f = int(counts[:, f].sum())
        if w.id_dist == "uniform":
            draws = rng.integers(0, w.cardinalities[f], size=n_f, dtype=np.int64)
        else:
            draws = bounded_zipf(rng, n_f, w.cardinalities[f], w.zipf_alpha, prefix)
        # scatter the draws of feature f to the token slots of its bags, in batch order
        pos = np.repeat(starts[:, f], counts[:, f]) + _ragged_arange(counts[:, f])
        ids[pos] = draws
    if sizes is None:
        return ids.reshape(B, F), None
    return ids, offsets


def _ragged_arange(counts: np.ndarray) -> np.ndarray:
    """concatenate(arange(c) for c in counts) without a Python loop."""
    total = int(counts.sum())
    if total == 0:
        return np.zeros(0, dtype=np.int64)
    ends = np.cumsum(counts)
    out = np.arange(total, dtype=np.int64)
    out -= np.repeat(ends - counts, counts)
    return out


def make_grad_out(w: Workload, seed: int = 2) -> np.ndarray:
    """float32[batch, F, d] ~ normal(0, 1) (tables of mixed dimensions: float32[batch, sum(dims)])."""
    rng = np.random.default_rng(seed)
    if w.dims is not None:
        return rng.standard_normal((w.batch, sum(w.dims)), dtype=np.float32)
    return rng.standard_normal((w.batch, w.n_features, w.d), dtype=np.float32)
