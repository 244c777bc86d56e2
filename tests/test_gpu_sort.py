"""The backward pass's radix sort on its own: against NumPy's stable sort of the
same key bits, element for element (keys and the values that travelled with
them), over sizes around the tile and wavefront boundaries, every number of
passes, partial last digits, and key distributions from all-equal to random."""
import numpy as np
import pytest
import torch

import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def check(keys: np.ndarray, lo: int, hi: int):
    n = keys.size
    vals = np.arange(n, dtype=np.uint32)[::-1].copy() if n else np.zeros(0, dtype=np.uint32)   # values unrelated to the order
    kd = torch.from_numpy(keys.view(np.int32).copy()).to(DEV)
    vd = torch.from_numpy(vals.view(np.int32).copy()).to(DEV)
    ks, vs = robe.robe_sort_pairs(kd, vd, lo, hi)
    got_k = ks.cpu().numpy().view(np.uint32)
    got_v = vs.cpu().numpy().view(np.uint32)
    digits = (keys.astype(np.uint64) >> np.uint64(lo)) & np.uint64((1 << (hi - lo)) - 1) if hi > lo else np.zeros(n, dtype=np.uint64)
    order = np.argsort(digits, kind="stable")
    assert np.array_equal(got_k, keys[order]), (n, lo, hi)
    assert np.array_equal(got_v, vals[order]), (n, lo, hi)


SIZES = [0, 1, 2, 63, 64, 65, 1023, 1024, 1025, 4095, 4096, 4097, 8192, 100_003, 1_000_001]
RANGES = [(0, 8), (0, 32), (7, 31), (15, 31), (23, 31), (3, 10), (0, 1), (31, 32), (5, 5), (4, 21)]


@pytest.mark.parametrize("n", SIZES)
def test_sorted_pairs_equal_numpys_stable_sort(n):
    rng = np.random.default_rng(n)
    keys = rng.integers(0, 2**32, size=n, dtype=np.uint64).astype(np.uint32)
    for lo, hi in RANGES:
        check(keys, lo, hi)


@pytest.mark.parametrize("kind", ["all equal", "two values", "few values", "sorted", "reversed", "low bits only"])
def test_key_distributions(kind):
    n = 300_007
    rng = np.random.default_rng(7)
    if kind == "all equal":
        keys = np.full(n, 0xDEADBEEF, dtype=np.uint32)
    elif kind == "two values":
        keys = rng.choice(np.array([5, 0x80000005], dtype=np.uint32), size=n)
    elif kind == "few values":
        keys = (rng.integers(0, 37, size=n, dtype=np.uint64) * 0x01010101 & 0xFFFFFFFF).astype(np.uint32)
    elif kind == "sorted":
        keys = np.sort(rng.integers(0, 2**31, size=n, dtype=np.uint64)).astype(np.uint32)
    elif kind == "reversed":
        keys = np.sort(rng.integers(0, 2**31, size=n, dtype=np.uint64))[::-1].astype(np.uint32)
    else:
        keys = rng.integers(0, 128, size=n, dtype=np.uint64).astype(np.uint32)
    for lo, hi in [(7, 31), (0, 32), (0, 8)]:
        check(keys, lo, hi)


def test_large_sort_and_bad_arguments():
    n = 9_000_001
    keys = np.random.default_rng(1).integers(0, 2**31, size=n, dtype=np.uint64).astype(np.uint32)
    check(keys, 7, 31)
    k = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(robe.RobeError):
        robe.robe_sort_pairs(k, k.clone(), 9, 8)
    with pytest.raises(robe.RobeError):
        robe.robe_sort_pairs(k, k.clone(), 0, 33)
    with pytest.raises(ValueError):
        robe.robe_sort_pairs(k, torch.zeros(3, dtype=torch.int32, device=DEV), 0, 8)
