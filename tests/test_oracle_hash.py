"""Pins for the oracle's integer maps: coefficient stream, h, g, idx.

Each test checks the C oracle against something other than itself: published
generator outputs, arbitrary-precision evaluation of the paper's formulas,
or a special case the paper names (Z = 1, Z = d, one fixed (e, c)).
"""
import os
import random

import numpy as np
import pytest

import oracle
from tests import brute

P = 2**31 - 1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_vectors.txt")


def _read_vectors():
    out, cur = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("seed"):
            cur = int(line.split()[1])
            out[cur] = []
        else:
            out[cur].append(int(line))
    return out


def test_splitmix64_matches_published_vectors():
    for seed, want in _read_vectors().items():
        assert oracle.splitmix64_stream(seed, len(want)) == want


def test_coefficients_follow_the_documented_recipe_and_ranges():
    # Section 3.2: multipliers in {1..P-1}, additive constants in {0..P-1}
    for seed in (0, 1, 42, 2**63 + 5, 2**64 - 1):
        H = oracle.init_hash(seed, 1000, 16, 4, 1)
        r = oracle.splitmix64_stream(seed, 8)
        want = tuple((v % P) if k in (3, 7) else 1 + v % (P - 1) for k, v in enumerate(r))
        assert H.coef == want
        for k, v in enumerate(H.coef):
            assert (0 if k in (3, 7) else 1) <= v <= P - 1
    assert oracle.init_hash(5, 1000, 16, 4, 1).coef == oracle.init_hash(5, 99, 8, 8, 0).coef
    assert oracle.init_hash(5, 1000, 16, 4, 1).coef != oracle.init_hash(6, 1000, 16, 4, 1).coef


EDGE_X = [0, 1, 2, P - 1, P, P + 1, 2 * P, 2**31, 2**32 - 1, 2**32, 2**62 - 1, 2**62, 2**63 - 1,
          -1, -2, -(2**63)]
EDGE_M = [1, 2, 3, 37, 1000, 2**20, 25_000_000, 250_000_000, 2**30, 2**31 - 2]


def test_h_and_g_equal_big_integer_evaluation():
    rnd = random.Random(1)
    for trial in range(40):
        m = EDGE_M[trial % len(EDGE_M)]
        H = oracle.init_hash(trial, m, 128, 1, 1)
        xs = EDGE_X + [rnd.randrange(0, 2**63) for _ in range(30)] + [rnd.randrange(0, 4 * 10**7) for _ in range(30)]
        for x in xs:
            e = rnd.randrange(0, 26)
            c = rnd.randrange(0, 128)
            hv = oracle.h(H, e, x, c)
            assert hv == brute.h(H.coef, P, m, e, x, c)
            assert 0 <= hv < m
            gv = oracle.g(H, e, x, c)
            assert gv == brute.g(H.coef, P, 1, e, x, c)
            assert gv in (-1, 1)


def test_h_with_extreme_coefficients():
    # coefficients at the ends of their ranges, where a 64-bit accumulator would wrap
    for coef in [(P - 1,) * 8, (1, 1, 1, 0, 1, 1, 1, 0), (P - 1, 1, P - 1, P - 1, 1, P - 1, 1, P - 1)]:
        H = oracle.Hash(2**31 - 2, 128, 1, 1, P, coef)
        for x in EDGE_X:
            for e, c in [(0, 0), (25, 127), (2**31 - 1, 2**20)]:
                assert oracle.h(H, e, x, c) == brute.h(coef, P, H.m, e, x, c)
                assert oracle.g(H, e, x, c) == brute.g(coef, P, 1, e, x, c)


def test_sign_off_gives_plus_one_and_sign_on_is_balanced():
    H0 = oracle.init_hash(3, 1000, 16, 4, 0)
    H1 = oracle.init_hash(3, 1000, 16, 4, 1)
    ids = np.arange(4000, dtype=np.int64)
    assert np.all(oracle.signs(H0, ids, 26) == 1)
    s = oracle.signs(H1, ids, 26)
    assert set(np.unique(s)) == {-1, 1}
    assert abs(float(s.mean())) < 0.05


def test_fixed_feature_and_chunk_reduces_to_one_key_universal_hash():
    # for one (e, c) the map is ((B x + b') mod P) mod m with b' = (A e + C c + D) mod P
    H = oracle.init_hash(11, 2**20, 16, 4, 0)
    A, B, C, D = H.coef[:4]
    for e, c in [(0, 0), (7, 3), (25, 1)]:
        b1 = (A * e + C * c + D) % P
        for x in [0, 1, 999, 123456789, 2**40 + 17]:
            assert oracle.h(H, e, x, c) == ((B * x + b1) % P) % H.m


def test_idx_is_chunk_offset_plus_position_with_wrap():
    # tiny arrays so that most blocks wrap (Section 3.2: the array is circular)
    rnd = random.Random(5)
    for (m, d, Z) in [(37, 16, 8), (8, 16, 8), (5, 20, 5), (64, 16, 4), (17, 16, 16), (3, 6, 1)]:
        H = oracle.init_hash(m * 131 + Z, m, d, Z, 0)
        wraps = 0
        for _ in range(60):
            e, x = rnd.randrange(0, 26), rnd.randrange(0, 10**6)
            pos = brute.position_map(H.coef, P, m, d, Z, e, x)
            got = [oracle.idx(H, e, x, i) for i in range(d)]
            assert got == pos
            for c in range(d // Z):
                blk = got[c * Z:(c + 1) * Z]
                assert len(set(blk)) == Z            # a block never collides with itself (Z <= m)
                wraps += blk[0] + Z > m
        if Z > 1:
            assert wraps > 0


def test_z_equal_one_is_per_element_hashing():
    # ROBE-1 (Section 3.3): every element is hashed on its own, idx(e,x,i) = h(e,x,i)
    H = oracle.init_hash(2, 1009, 16, 1, 0)
    for e, x in [(0, 0), (3, 77), (25, 10**9)]:
        for i in range(16):
            assert oracle.idx(H, e, x, i) == oracle.h(H, e, x, i) == brute.h(H.coef, P, H.m, e, x, i)


def test_z_equal_d_is_one_circular_slice():
    # ROBE-D (Section 3.1): the whole embedding starts at h(e,x) and continues, wrapping
    H = oracle.init_hash(9, 203, 16, 16, 0)
    for e, x in [(0, 5), (1, 6), (25, 12345), (4, 2**50)]:
        start = brute.h(H.coef, P, H.m, e, x, 0)
        assert [oracle.idx(H, e, x, i) for i in range(16)] == [(start + i) % H.m for i in range(16)]


def test_block_larger_than_embedding_follows_the_flattened_table():
    # Z > d (Section 3.3): the flattened table cut into chunks of Z; r = Z/d embeddings share a chunk
    rnd = random.Random(9)
    for (m, d, Z) in [(1000, 4, 16), (37, 4, 16), (32, 8, 32), (100_003, 16, 64), (4099, 8, 24), (50, 1, 7)]:
        H = oracle.init_hash(m + Z, m, d, Z, 0)
        r = Z // d
        for x in [0, 1, r - 1, r, r + 1, 12345, 2**40 + 3, 2**63 - 1, -1] + [rnd.randrange(0, 10**7) for _ in range(40)]:
            e = rnd.randrange(0, 26)
            got = [oracle.idx(H, e, x, i) for i in range(d)]
            assert got == [brute.position_big_block(H.coef, P, m, d, Z, e, x, i) for i in range(d)]
            assert got == [(got[0] + i) % m for i in range(d)]          # an embedding stays contiguous
        # tokens of one chunk lie side by side, d apart; the next chunk starts somewhere else
        base = [oracle.idx(H, 3, r * 5 + k, 0) for k in range(r)]
        assert base == [(base[0] + k * d) % m for k in range(r)]
    H = oracle.init_hash(1, 1000, 4, 16, 0)
    flat = np.array([5, 6, 7, 8, 9], dtype=np.int64)
    off = oracle.offsets(H, flat, 2)
    assert off.shape == (5, 1)
    assert off[:, 0].tolist() == [oracle.idx(H, k % 2, int(flat[k]), 0) for k in range(5)]


def test_batched_offsets_and_signs_agree_with_scalar_calls():
    H = oracle.init_hash(21, 25_000_000, 128, 32, 1)
    rnd = np.random.default_rng(0)
    ids = rnd.integers(0, 4 * 10**7, size=(5, 26))
    off = oracle.offsets(H, ids, 26)
    sg = oracle.signs(H, ids, 26)
    flat = ids.ravel()
    for k in range(flat.size):
        for c in range(4):
            assert off[k, c] == brute.h(H.coef, P, H.m, k % 26, int(flat[k]), c)
        for i in (0, 1, 31, 32, 127):
            assert sg[k, i] == brute.g(H.coef, P, 1, k % 26, int(flat[k]), i)


def test_rejects_bad_shapes():
    for (m, d, Z) in [(0, 16, 4), (100, 16, 5), (100, 0, 1), (100, 16, 0), (8, 16, 16)]:
        with pytest.raises(ValueError):
            oracle.init_hash(0, m, d, Z, 0)
