"""GPU parity for tables of different dimensions sharing the array (Section 3.2,
"Multiple embedding tables"): robe_forward_mixed / robe_backward_mixed against
the oracle's mixed functions, element by element, on seeded synthetic inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TINY = 1e-30


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits_equal(a, b):
    return np.array_equal(np.ascontiguousarray(a).ravel().view(np.int32), np.ascontiguousarray(b).ravel().view(np.int32))


def hashes(seed, m, Z, sign, dmax):
    h = robe.robe_init_hash(seed, m, dmax, Z, sign)
    H = oracle.init_hash(seed, m, dmax, Z, sign)
    assert tuple(h.coef) == H.coef
    return h, H


# (m, dims, Z): runs of equal dimensions, alternating ones, every lane layout, a dimension only the
# shape-generic kernel takes (12 with Z = 3 -> 24), rows whose starts are not 16-byte aligned (Z = 1,
# odd dimensions), an array small enough that blocks wrap
CASES = [
    (1_000_003, (128, 128, 64, 64, 64, 32, 128), 32),
    (100_003, (16, 4, 4, 8, 16, 16, 4), 4),
    (70_001, (8, 16, 8, 16, 8, 16), 8),
    (9973, (3, 12, 24, 3, 6), 3),
    (4099, (1, 5, 2, 7, 64, 1), 1),
    (61, (16, 8, 8, 32), 8),
    (500_009, (256, 512, 128), 128),
    (100_003, (4, 16, 64, 8, 16, 2), 16),       # tables narrower than the block: 4, 2 and 8 tokens share one (Section 3.3)
    (70_001, (1, 3, 6, 12), 6),
    (200_003, tuple(8 * (1 + k % 4) for k in range(70)), 8),      # more tables than one launch's table map holds
]
ROUTES = [robe.ROUTE_DIRECT, robe.ROUTE_COMBINE, robe.ROUTE_REGIONS]


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,dims,Z", CASES)
def test_mixed_single_hot_forward_is_bit_exact_and_backward_within_tolerance(m, dims, Z, sign, route):
    opt = robe.options(backward_route=route)
    h, H = hashes(7 * m + Z + sign, m, Z, sign, max(dims))
    F, B = len(dims), 257
    rng = np.random.default_rng(m + sum(dims))
    ids = rng.integers(0, 5000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.2] = 3
    M = rng.standard_normal(m).astype(np.float32)
    out = robe.robe_forward_mixed(h, dims, dev(M), dev(ids), None, B).cpu().numpy()
    assert bits_equal(out, oracle.forward_mixed(H, dims, M, ids, None, B))
    G = rng.standard_normal((B, sum(dims))).astype(np.float32)
    ga = torch.zeros(m, dtype=torch.float32, device=DEV)
    sorted_route = route != robe.ROUTE_DIRECT and min(dims) >= Z and max(dims) <= 512
    assert (robe.robe_mixed_workspace_bytes(h, dims, B, ids.size, opt) > 0) == sorted_route
    robe.robe_backward_mixed(h, dims, dev(G), dev(ids), None, B, ga, options=opt)
    ref, S = oracle.backward_mixed(H, dims, G, ids, None, B)
    got = ga.cpu().numpy()
    assert np.all(np.abs(got.astype(np.float64) - ref) <= 1e-5 * S + TINY)
    assert not got[S == 0].any()
    # accumulates onto what is there
    robe.robe_backward_mixed(h, dims, dev(G), dev(ids), None, B, ga, options=opt)
    assert np.all(np.abs(ga.cpu().numpy().astype(np.float64) - 2 * ref) <= 2e-5 * S + TINY)
    # small-integer gradients: exact in any order
    Gi = rng.integers(-3, 4, size=(B, sum(dims))).astype(np.float32)
    ga.zero_()
    robe.robe_backward_mixed(h, dims, dev(Gi), dev(ids), None, B, ga, options=opt)
    refi, _ = oracle.backward_mixed(H, dims, Gi, ids, None, B)
    assert np.array_equal(ga.cpu().numpy().astype(np.float64), refi)


@pytest.mark.parametrize("route", ROUTES)
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,dims,Z", CASES)
def test_mixed_bags_within_tolerance(m, dims, Z, sign, route):
    opt = robe.options(backward_route=route)
    h, H = hashes(11 * m + Z + sign, m, Z, sign, max(dims))
    F, B = len(dims), 131
    rng = np.random.default_rng(m + 1)
    sizes = rng.poisson(4.0, size=B * F).astype(np.int64)
    sizes[0] = 0
    sizes[5] = 70
    off = np.zeros(B * F + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    flat = rng.integers(0, 3000, size=int(off[-1]), dtype=np.int64)
    M = rng.standard_normal(m).astype(np.float32)
    out = robe.robe_forward_mixed(h, dims, dev(M), dev(flat), dev(off), B).cpu().numpy()
    want = oracle.forward_mixed(H, dims, M, flat, off, B)
    H_abs = oracle.Hash(H.m, H.d, H.Z, 0, H.P, H.coef)
    S = oracle.forward_mixed(H_abs, dims, np.abs(M), flat, off, B).astype(np.float64)
    assert np.all(np.abs(out.astype(np.float64) - want) <= 1e-5 * S + TINY)
    G = rng.standard_normal((B, sum(dims))).astype(np.float32)
    ga = torch.zeros(m, dtype=torch.float32, device=DEV)
    robe.robe_backward_mixed(h, dims, dev(G), dev(flat), dev(off), B, ga, options=opt)
    ref, Sb = oracle.backward_mixed(H, dims, G, flat, off, B)
    assert np.all(np.abs(ga.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * Sb + TINY)


def test_mixed_with_equal_dimensions_is_the_plain_forward_bitwise():
    h, H = hashes(5, 250_007, 32, 1, 128)
    rng = np.random.default_rng(5)
    B, F = 300, 26
    ids = rng.integers(0, 10**6, size=(B, F), dtype=np.int64)
    M = rng.standard_normal(250_007).astype(np.float32)
    a = robe.robe_forward_mixed(h, [128] * F, dev(M), dev(ids), None, B).cpu().numpy()
    b = robe.robe_forward(h, dev(M), dev(ids), None, B, F).cpu().numpy()
    assert bits_equal(a, b)


def test_mixed_rejects_bad_dimensions_and_what_the_reproducible_option_cannot_do():
    h, _ = hashes(1, 1000, 4, 0, 16)
    ids = dev(np.zeros((2, 3), dtype=np.int64))
    M = torch.zeros(1000, dtype=torch.float32, device=DEV)
    for dims in ([16, 6, 4], [16, 0, 4], [3, 4, 4]):
        with pytest.raises(robe.RobeError) as ei:
            robe.robe_forward_mixed(h, dims, M, ids, None, 2)
        assert ei.value.code == robe.ROBE_EINVAL
    # a table narrower than the block has no route without float atomics: a loud error
    opt = robe.options(reproducible=1)
    with pytest.raises(robe.RobeError) as ei:
        robe.robe_backward_mixed(h, [16, 2, 4], torch.zeros((2, 22), dtype=torch.float32, device=DEV), ids, None, 2, M,
                                 options=opt)
    assert ei.value.code == robe.ROBE_EINVAL and "reproducible" in str(ei.value)
    with pytest.raises(robe.RobeError):
        robe.robe_mixed_workspace_bytes(h, [16, 2, 4], 2, 6, opt)
    with pytest.raises(robe.RobeError):
        robe.robe_backward_adagrad_mixed(h, [16, 2, 4], torch.zeros((2, 22), dtype=torch.float32, device=DEV), ids, None, 2,
                                         M, torch.zeros_like(M), 0.01, 1e-8, options=opt)
    assert robe.robe_forward_mixed(h, [16, 4, 4], M, dev(np.zeros((0, 3), dtype=np.int64)), None, 0).shape == (0, 24)


def _fused_mixed_check(h, H, dims, Gi, ids, off, B, m, opt):
    """robe_backward_adagrad_mixed against oracle.backward_mixed -> oracle.adagrad; small-integer
    gradients make every slot's sum exact, so both sides feed the same gradient to the update."""
    rng = np.random.default_rng(m + B)
    M0 = rng.standard_normal(m).astype(np.float32)
    s0 = (rng.random(m) * (rng.random(m) < 0.5)).astype(np.float32)
    Md, sd = dev(M0), dev(s0)
    robe.robe_backward_adagrad_mixed(h, dims, dev(Gi), dev(ids), dev(off), B, Md, sd, 0.01, 1e-8, options=opt)
    g, _ = oracle.backward_mixed(H, dims, Gi, ids, off, B)
    assert np.array_equal(g, np.round(g))
    Mo, so, go = M0.copy(), s0.copy(), g.astype(np.float32)
    oracle.adagrad(Mo, so, go, 0.01, 1e-8)
    Mg, sg = Md.cpu().numpy(), sd.cpu().numpy()
    untouched = g == 0
    assert bits_equal(Mg[untouched], M0[untouched]) and bits_equal(sg[untouched], s0[untouched])
    step = np.abs(Mo.astype(np.float64) - M0)
    assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(M0) + step) + TINY)
    assert np.all(np.abs(sg.astype(np.float64) - so) <= 1e-6 * np.abs(so) + TINY)
    assert not bits_equal(Mg, M0)


# (m, dims, Z, options of the fused call).  Region route with record kernels (small arrays), with the
# lookup in the sorted list (large arrays: region_records = 2), the two-step fallback (a table
# narrower than the block; a small array by default), regions of 2^10 floats.
FUSED = [
    (1_000_003, (128, 128, 64, 64, 64, 32, 128), 32, dict(fused_route=robe.ROUTE_REGIONS)),
    (3_000_017, (8, 32, 8, 16, 4, 64), 4, dict(fused_route=robe.ROUTE_REGIONS, region_shift=10)),
    (2**27 + 3, (64, 32, 64, 64, 32), 32, dict(region_records=2)),
    (45_000_007, (64, 32, 32, 64), 32, dict(fused_route=robe.ROUTE_REGIONS, region_records=2)),
    (100_003, (4, 16, 64, 8, 16, 2), 16, dict()),
    (500_009, (256, 512, 128), 128, dict()),
    (500_009, (256, 512, 128), 128, dict(fused_route=robe.ROUTE_REGIONS)),
]


@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,dims,Z,fields", FUSED)
def test_fused_mixed_step_matches_the_oracle(m, dims, Z, fields, sign):
    opt = robe.options(**fields)
    h, H = hashes(13 * m + Z + sign, m, Z, sign, max(dims))
    F, B = len(dims), 900
    rng = np.random.default_rng(m % 1000 + Z)
    ids = rng.integers(0, 20_000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.25] = 3                          # one token hundreds of times in every table
    Gi = rng.integers(-3, 4, size=(B, sum(dims))).astype(np.float32)
    regions = fields.get("fused_route") == robe.ROUTE_REGIONS or m >= 2**26
    need = robe.robe_fused_mixed_workspace_bytes(h, dims, B, ids.size, opt)
    assert (need < 4 * m) == (regions and min(dims) >= Z)       # the fused route needs no gradient array
    _fused_mixed_check(h, H, dims, Gi, ids, None, B, m, opt)
    # bags, one of them long
    Bb = 150
    sizes = rng.poisson(5.0, size=Bb * F).astype(np.int64)
    sizes[3] = 400
    off = np.zeros(Bb * F + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    flat = rng.integers(0, 5000, size=int(off[-1]), dtype=np.int64)
    _fused_mixed_check(h, H, dims, Gi[:Bb], flat, off, Bb, m, opt)


@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,dims,Z,records", [(1_000_003, (128, 64, 32, 128, 64), 32, 0), (2**27 + 3, (64, 32, 64, 32), 32, 2),
                                              (20_011, (32, 8, 16, 8), 8, 0)])
def test_mixed_reproducible_option_gives_the_same_bits_every_run(m, dims, Z, records, sign):
    opt = robe.options(reproducible=1, region_records=records)
    h, H = hashes(3 * m + Z + sign, m, Z, sign, max(dims))
    F, B = len(dims), 3000
    rng = np.random.default_rng(m % 777)
    ids = rng.integers(0, 30_000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.2] = 7
    G = rng.standard_normal((B, sum(dims))).astype(np.float32)
    M0 = rng.standard_normal(m).astype(np.float32)
    Gd, idd = dev(G), dev(ids)
    assert robe.robe_mixed_workspace_bytes(h, dims, B, ids.size, opt) > 8 * ids.size
    runs = []
    for _ in range(3):
        Md, sd = dev(M0), torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward_adagrad_mixed(h, dims, Gd, idd, None, B, Md, sd, 0.01, 1e-8, options=opt)
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward_mixed(h, dims, Gd, idd, None, B, ga, options=opt)
        runs.append((Md.cpu().numpy(), sd.cpu().numpy(), ga.cpu().numpy()))
    for Mk, sk, gk in runs[1:]:
        assert bits_equal(Mk, runs[0][0]) and bits_equal(sk, runs[0][1]) and bits_equal(gk, runs[0][2])
    ref, S = oracle.backward_mixed(H, dims, G, ids, None, B)
    assert np.all(np.abs(runs[0][2].astype(np.float64) - ref) <= 1e-5 * S + TINY)
    # the accumulator of the fused call is the square of the very gradient the plain call returns
    g32 = runs[0][2]
    assert bits_equal(runs[0][1], g32 * g32)


def test_mixed_sorted_route_keeps_equal_keys_of_different_tables_apart():
    # Two tables of different dimension whose tokens share a sort key: with 8 key bits nearly all
    # neighbours in the sorted list do.  A run must end where the table changes even if the key does not.
    m, Z, dims = 200_003, 4, (8, 32, 8, 16, 4, 64)
    h, H = hashes(9, m, Z, 0, max(dims))
    B = 700
    rng = np.random.default_rng(1)
    ids = rng.integers(0, 30, size=(B, len(dims)), dtype=np.int64)
    Gi = rng.integers(-3, 4, size=(B, sum(dims))).astype(np.float32)
    for kb, route in ((8, robe.ROUTE_COMBINE), (31, robe.ROUTE_COMBINE), (8, robe.ROUTE_REGIONS), (31, robe.ROUTE_REGIONS)):
        opt = robe.options(backward_route=route, key_bits=kb)
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward_mixed(h, dims, dev(Gi), dev(ids), None, B, ga, options=opt)
        ref, _ = oracle.backward_mixed(H, dims, Gi, ids, None, B)
        assert np.array_equal(ga.cpu().numpy().astype(np.float64), ref), (kb, route)
