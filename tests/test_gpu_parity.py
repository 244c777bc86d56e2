"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Bars (from the workload statement): hash offsets, signs and single-hot forward
are bit-exact; pooled forward and the atomic backward agree within
1e-5 * S + tiny, where S is the sum of |term| over the terms of that output
element (a backward-error bound: plain relative error is ill-posed where
terms cancel); Adagrad on identical inputs agrees within 1e-6 of the
magnitudes involved.  Integer-valued gradients make float32 sums exact in any
order, which gives a bit-exact backward test as well.
"""
import ctypes
import os

import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2108_02191_amd as robe

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
THREADS = max(1, min(16, os.cpu_count() or 1))
TINY = 1e-30


def to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


ROUTES = {"direct": robe.ROUTE_DIRECT, "dedup": robe.ROUTE_COMBINE, "regions": robe.ROUTE_REGIONS}


def both_hashes(seed, m, d, Z, sign):
    h = robe.robe_init_hash(seed, m, d, Z, sign)
    H = oracle.init_hash(seed, m, d, Z, sign)
    assert tuple(h.coef) == H.coef
    return h, H


def bits_equal(a, b):
    a = np.ascontiguousarray(a, dtype=np.float32).ravel().view(np.int32)
    b = np.ascontiguousarray(b, dtype=np.float32).ravel().view(np.int32)
    return np.array_equal(a, b)


def random_bags(rng, rows, card, mean, long_bag=0):
    sizes = rng.poisson(mean, size=rows).astype(np.int64)
    sizes[0] = 0
    if rows > 3:
        sizes[rows // 2] = 0
        sizes[3] = long_bag or sizes[3]
    off = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    ids = rng.integers(0, card, size=int(off[-1]), dtype=np.int64)
    return ids, off


# (m, d, Z): every lane layout (1/2/4 elements per lane, consecutive and strided; 3/6/8 strided: d = 6,
# 12, 24, 48, 96, 192, 384, 512; lane groups wider than the row: d = 5, 100), the shape-generic kernel
# (d > 512), arrays small enough that blocks wrap, Z = m, Z = 1, Z = d, Z > d.
SHAPES = [
    (2**20, 16, 4), (1_000_003, 128, 32), (999_983, 128, 8), (500_000, 128, 128), (300_007, 128, 1),
    (37, 16, 8), (16, 16, 16), (64, 64, 64), (101, 8, 2), (50, 4, 1), (1000, 6, 2),
    (70_001, 96, 32), (4099, 12, 3), (9973, 256, 32), (100_000, 512, 128), (5, 5, 5), (1, 1, 1),
    (50_021, 384, 64), (33_331, 192, 48), (20_011, 48, 16), (9001, 24, 24), (777, 512, 1), (100_003, 100, 10),
    (60_013, 120, 40), (30_011, 80, 80), (200_003, 640, 64), (5003, 513, 27),
    (1000, 4, 16), (37, 4, 16), (32, 8, 32), (100_003, 16, 64), (4099, 8, 24), (250_007, 128, 512),   # Z > d
    (2**31 - 1, 32, 16),
]


@pytest.mark.parametrize("m,d,Z", SHAPES)
def test_offsets_and_signs_are_bit_exact(m, d, Z):
    h, H = both_hashes(m + d, m, d, Z, 1)
    rng = np.random.default_rng(m)
    F = 26
    ids = np.concatenate([
        rng.integers(0, 4 * 10**7, size=3000, dtype=np.int64),
        rng.integers(0, 2**63 - 1, size=500, dtype=np.int64),
        np.array([0, 1, 2**31 - 2, 2**31 - 1, 2**31, 2**32 - 1, 2**32, 2**62, 2**63 - 1, -1, -2, -(2**63)], dtype=np.int64),
    ])
    off, sg = robe.robe_offsets(h, to_dev(ids), F, want_signs=True)
    assert np.array_equal(off.cpu().numpy(), oracle.offsets(H, ids, F))
    assert np.array_equal(sg.cpu().numpy(), oracle.signs(H, ids, F))


@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z", SHAPES[:-1])
def test_single_hot_forward_is_bit_exact(m, d, Z, sign):
    h, H = both_hashes(11 * m + Z, m, d, Z, sign)
    B, F = 37, 26                                   # 962 rows: several wavefront tiles and a ragged tail
    rng = np.random.default_rng(d * 7 + Z)
    ids = rng.integers(0, 5000, size=(B, F), dtype=np.int64)
    M = workloads.make_array(m, 3)
    if m > 8:
        M[::7] = -0.0                               # signed zeros must survive the copy
    out = robe.robe_forward(h, to_dev(M), to_dev(ids), None, B, F)
    assert bits_equal(out.cpu().numpy(), oracle.forward(H, M, ids, None, B, F, threads=THREADS))


def test_single_hot_forward_huge_array_bit_exact():
    m, d, Z = 2**31 - 1, 32, 16                    # largest legal array: 8 GiB of float32
    h, H = both_hashes(5, m, d, Z, 1)
    B, F = 64, 26
    ids = np.random.default_rng(0).integers(0, 2**40, size=(B, F), dtype=np.int64)
    M = torch.empty(m, dtype=torch.float32, device=DEV)
    M.copy_(torch.arange(m, device=DEV, dtype=torch.int32).bitwise_and_(0xFFFFF).to(torch.float32))
    out = robe.robe_forward(h, M, to_dev(ids), None, B, F).cpu().numpy()
    # oracle on the positions only: value at slot j is (j & 0xFFFFF)
    off = oracle.offsets(H, ids, F)
    sg = oracle.signs(H, ids, F)
    i = np.arange(d)
    pos = (off[:, i // Z] + (i % Z)[None, :]) % m
    want = (pos & 0xFFFFF).astype(np.float32) * sg
    assert bits_equal(out.reshape(-1, d), want)
    del M
    torch.cuda.empty_cache()


@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z", SHAPES[:-1])
def test_bag_forward_within_tolerance(m, d, Z, sign):
    h, H = both_hashes(13 * m + Z, m, d, Z, sign)
    B, F = 19, 26
    rng = np.random.default_rng(d + Z)
    ids, off = random_bags(rng, B * F, 3000, 6.0, long_bag=333)
    M = workloads.make_array(m, 4)
    out = robe.robe_forward(h, to_dev(M), to_dev(ids), to_dev(off), B, F).cpu().numpy()
    want = oracle.forward(H, M, ids, off, B, F, threads=THREADS)
    H_abs = oracle.Hash(H.m, H.d, H.Z, 0, H.P, H.coef)
    S = oracle.forward(H_abs, np.abs(M), ids, off, B, F, threads=THREADS).astype(np.float64)
    err = np.abs(out.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= 1e-5 * S + TINY), float((err / (S + TINY)).max())
    empty = np.diff(off) == 0
    assert empty.any()
    flat = out.reshape(B * F, d)
    assert not flat[empty].any() and not np.signbit(flat[empty]).any()


def test_bag_of_one_token_equals_single_hot_bitwise():
    w = workloads.get("tiny")
    h, H = both_hashes(3, 100_003, 128, 32, 1)
    B, F = 50, w.n_features
    ids = np.random.default_rng(1).integers(0, 10**6, size=(B, F), dtype=np.int64)
    M = to_dev(workloads.make_array(100_003, 1))
    single = robe.robe_forward(h, M, to_dev(ids), None, B, F)
    bags = robe.robe_forward(h, M, to_dev(ids.ravel()), to_dev(np.arange(B * F + 1, dtype=np.int64)), B, F)
    # a bag sum starts from +0.0, so only a -0.0 could differ; the array has none
    assert bits_equal(single.cpu().numpy(), bags.cpu().numpy())


def check_backward(h, H, G, ids, off, B, F, options=None):
    ga = torch.zeros(H.m, dtype=torch.float32, device=DEV)
    robe.robe_backward(h, to_dev(G), to_dev(ids), to_dev(off), B, F, ga, options=options)
    got = ga.cpu().numpy().astype(np.float64)
    want, S = oracle.backward(H, G, ids, off, B, F, threads=1)
    err = np.abs(got - want)
    assert np.all(err <= 1e-5 * S + TINY), float((err / (S + TINY)).max())
    assert np.all(got[S == 0] == 0)                  # untouched slots stay zero
    return got, want


@pytest.mark.parametrize("mode", ["direct", "dedup", "regions"])
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z", SHAPES[:-1])
def test_backward_single_hot_and_bags(m, d, Z, sign, mode):
    # every scatter strategy: per-element atomics, duplicates combined first, and the region route
    # (shapes a sorted route cannot take fall back to the atomics)
    opt = robe.options(backward_route=ROUTES[mode])
    h, H = both_hashes(17 * m + Z, m, d, Z, sign)
    B, F = 23, 26
    rng = np.random.default_rng(d * 3 + Z)
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    ids = rng.integers(0, 40, size=(B, F), dtype=np.int64)     # few tokens: heavy collisions
    check_backward(h, H, G, ids, None, B, F, opt)
    idsb, off = random_bags(rng, B * F, 200, 5.0, long_bag=150)
    check_backward(h, H, G, idsb, off, B, F, opt)
    # small-integer gradients: float32 sums are exact in any order -> bit-exact scatter
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    got, want = check_backward(h, H, Gi, idsb, off, B, F, opt)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("tile,xcd", [(2, robe.ROWS_MEMORY), (2, robe.ROWS_BY_TABLE_ALWAYS), (1, robe.ROWS_MEMORY),
                                      (1, robe.ROWS_BY_TABLE_ALWAYS)])
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z,B,F", [(1_000_003, 128, 32, 700, 26), (100_003, 16, 4, 2048, 26), (37, 16, 8, 300, 5),
                                       (70_001, 64, 64, 129, 3), (4099, 8, 1, 1000, 7), (9973, 256, 32, 65, 2),
                                       (999_983, 2, 2, 5000, 26), (500, 1, 1, 200, 1)])
def test_direct_single_hot_backward_with_and_without_tile_combining(m, d, Z, B, F, sign, tile, xcd):
    # the direct scatter: tiles of 64 lookups with their duplicates combined (in memory order and
    # walked table by table), and the plain one-atomic-per-element kernel; tables of 3 to 10^6 tokens
    opt = robe.options(backward_route=robe.ROUTE_DIRECT, tile_combine=tile, row_order=xcd)
    h, H = both_hashes(29 * m + Z + sign, m, d, Z, sign)
    rng = np.random.default_rng(m + B)
    card = np.array([3, 10, 1000, 10**6] * 7)[:F]
    ids = (rng.integers(0, 2**40, size=(B, F)) % card).astype(np.int64)
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    check_backward(h, H, G, ids, None, B, F, opt)
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    got, want = check_backward(h, H, Gi, ids, None, B, F, opt)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("mode", ["direct", "dedup", "regions"])
def test_backward_accumulates_onto_existing_values(mode):
    opt = robe.options(backward_route=ROUTES[mode])
    h, H = both_hashes(2, 50_021, 16, 4, 0)
    B, F = 8, 26
    rng = np.random.default_rng(0)
    ids = rng.integers(0, 1000, size=(B, F), dtype=np.int64)
    G = rng.integers(-2, 3, size=(B, F, 16)).astype(np.float32)
    ga = torch.full((H.m,), 5.0, dtype=torch.float32, device=DEV)
    robe.robe_backward(h, to_dev(G), to_dev(ids), None, B, F, ga, options=opt)
    robe.robe_backward(h, to_dev(G), to_dev(ids), None, B, F, ga, options=opt)
    want, _ = oracle.backward(H, G, ids, None, B, F)
    assert np.array_equal(ga.cpu().numpy().astype(np.float64), 5.0 + 2 * want)


@pytest.mark.parametrize("mode,rshift", [("dedup", 0), ("regions", 0), ("regions", 10), ("regions", 15)])
@pytest.mark.parametrize("key_bits", [31, 16, 8])
@pytest.mark.parametrize("sign", [0, 1])
def test_dedup_backward_hot_tokens_and_key_collisions(key_bits, sign, mode, rshift):
    # one token repeated thousands of times (runs far longer than a lane group's stretch), a coarse
    # sort key so that distinct tokens share keys and interleave, blocks that wrap or leave their
    # region, unaligned grad_array; with float atomics and with the region-sorted scatter
    opt = robe.options(backward_route=ROUTES[mode], region_shift=rshift, key_bits=key_bits)
    m, d, Z, B, F = 100_003, 64, 32, 301, 7
    h, H = both_hashes(31 + key_bits, m, d, Z, sign)
    rng = np.random.default_rng(key_bits)
    ids = rng.integers(0, 5000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.6] = 7                            # the hot token
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    for shift in (0, 1):
        buf = torch.zeros(m + shift, dtype=torch.float32, device=DEV)
        ga = buf[shift:]
        assert robe.robe_workspace_bytes(h, B, F, ids.size, opt) > 0
        robe.robe_backward(h, to_dev(Gi), to_dev(ids), None, B, F, ga, options=opt)
        want, _ = oracle.backward(H, Gi, ids, None, B, F)
        assert np.array_equal(ga.cpu().numpy().astype(np.float64), want)
    idsb, off = random_bags(rng, B * F, 30, 9.0, long_bag=5000)
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    check_backward(h, H, G, idsb, off, B, F, opt)


def test_dedup_backward_needs_its_workspace():
    w = workloads.get("training").scaled(batch=16384)            # 54 M element updates: above the size where sorting pays
    h = robe.robe_init_hash(1, w.m, w.d, w.Z, 0)
    n = w.batch * w.n_features
    need = robe.robe_workspace_bytes(h, w.batch, w.n_features, n)
    assert need >= 16 * n                                        # two (key, position) buffers of 4-byte entries
    ids = torch.zeros((w.batch, w.n_features), dtype=torch.int64, device=DEV)
    G = torch.zeros((w.batch, w.n_features, w.d), dtype=torch.float32, device=DEV)
    ga = torch.zeros(w.m, dtype=torch.float32, device=DEV)
    small = torch.empty(need // 2, dtype=torch.uint8, device=DEV)
    rc = robe.lib().robe_backward(ctypes.byref(h), G.data_ptr(), ids.data_ptr(), None, n, w.batch, w.n_features,
                                  ga.data_ptr(), small.data_ptr(), need // 2, None, None)
    assert rc == robe.ROBE_EINVAL and b"workspace" in robe.lib().robe_last_error()
    rc = robe.lib().robe_backward(ctypes.byref(h), G.data_ptr(), ids.data_ptr(), None, n, w.batch, w.n_features,
                                  ga.data_ptr(), None, 0, None, None)
    assert rc == robe.ROBE_EINVAL


@pytest.mark.parametrize("m,shift", [(4096, 0), (4099, 0), (4099, 1), (3, 0), (1, 0), (1_000_001, 3)])
def test_adagrad_matches_oracle_and_leaves_untouched_slots_alone(m, shift):
    rng = np.random.default_rng(m + shift)
    h = robe.robe_init_hash(0, m, 1, 1, 0)
    M0 = rng.standard_normal(m).astype(np.float32)
    s0 = (rng.random(m).astype(np.float32)) * (rng.random(m) < 0.7)
    g0 = rng.standard_normal(m).astype(np.float32) * (rng.random(m) < 0.6)
    # `shift` floats of padding in front put the buffers off 16-byte alignment (scalar kernel)
    def dev(a):
        buf = torch.zeros(m + shift, dtype=torch.float32, device=DEV)
        view = buf[shift:]
        view.copy_(torch.from_numpy(a))
        return view
    M, s, g = dev(M0), dev(s0), dev(g0)
    robe.robe_adagrad_update(h, M, s, g, 0.01, 1e-8)
    Mo, so, go = M0.copy(), s0.copy(), g0.copy()
    oracle.adagrad(Mo, so, go, 0.01, 1e-8)
    Mg, sg = M.cpu().numpy(), s.cpu().numpy()
    assert not g.cpu().numpy().any()
    untouched = g0 == 0
    assert bits_equal(Mg[untouched], M0[untouched]) and bits_equal(sg[untouched], s0[untouched])
    step = np.abs(Mo.astype(np.float64) - M0)
    assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(M0) + step) + TINY)
    assert np.all(np.abs(sg.astype(np.float64) - so) <= 1e-6 * np.abs(so) + TINY)
    assert untouched.all() or not bits_equal(Mg, M0)


@pytest.mark.parametrize("m,shift", [(4096, 0), (4099, 1), (3, 0), (1_000_001, 2)])
def test_sgd_matches_oracle_and_leaves_untouched_slots_alone(m, shift):
    rng = np.random.default_rng(m + shift)
    h = robe.robe_init_hash(0, m, 1, 1, 0)
    M0 = rng.standard_normal(m).astype(np.float32)
    g0 = rng.standard_normal(m).astype(np.float32) * (rng.random(m) < 0.6)
    def dev(a):
        buf = torch.zeros(m + shift, dtype=torch.float32, device=DEV)
        view = buf[shift:]
        view.copy_(torch.from_numpy(a))
        return view
    M, g = dev(M0), dev(g0)
    robe.robe_sgd_update(h, M, g, 1.0)
    Mo, go = M0.copy(), g0.copy()
    oracle.sgd(Mo, go, 1.0)
    Mg = M.cpu().numpy()
    assert not g.cpu().numpy().any()
    assert bits_equal(Mg[g0 == 0], M0[g0 == 0])
    # float32 multiply then subtract (two roundings) against one rounding of the exact value
    assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(M0) + np.abs(g0)) + TINY)
    # with lr = 1 the product is exact, so the result is the correctly rounded difference: bit-exact
    assert bits_equal(Mg, Mo)


def _check_fused(h, H, Gi, ids, off, B, F, m, shift=0, options=None):
    """Fused backward + Adagrad against oracle.backward -> oracle.adagrad.  Small-integer gradients
    make every slot's sum exact, so both sides feed the same gradient to the update."""
    rng = np.random.default_rng(m + B)
    M0 = rng.standard_normal(m).astype(np.float32)
    s0 = (rng.random(m) * (rng.random(m) < 0.5)).astype(np.float32)
    def dev_view(a):
        buf = torch.zeros(m + shift, dtype=torch.float32, device=DEV)
        view = buf[shift:]
        view.copy_(torch.from_numpy(a))
        return view
    Md, sd = dev_view(M0), dev_view(s0)
    robe.robe_backward_adagrad(h, to_dev(Gi), to_dev(ids), to_dev(off), B, F, Md, sd, 0.01, 1e-8, options=options)
    g, _ = oracle.backward(H, Gi, ids, off, B, F)
    assert np.array_equal(g, np.round(g))
    Mo, so, go = M0.copy(), s0.copy(), g.astype(np.float32)
    oracle.adagrad(Mo, so, go, 0.01, 1e-8)
    Mg, sg = Md.cpu().numpy(), sd.cpu().numpy()
    untouched = g == 0
    assert bits_equal(Mg[untouched], M0[untouched]) and bits_equal(sg[untouched], s0[untouched])
    step = np.abs(Mo.astype(np.float64) - M0)
    assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(M0) + step) + TINY)
    assert np.all(np.abs(sg.astype(np.float64) - so) <= 1e-6 * np.abs(so) + TINY)
    assert untouched.all() or not bits_equal(Mg, M0)


@pytest.mark.parametrize("route", [robe.ROUTE_REGIONS, robe.ROUTE_TWO_STEP, robe.ROUTE_AUTO])
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z,records", [(1_000_003, 128, 32, 0), (2**26 + 3, 64, 32, 2), (1000, 64, 32, 0), (100_003, 16, 64, 0)])
def test_fused_backward_sgd_matches_backward_then_sgd(m, d, Z, records, sign, route):
    # robe_backward_sgd against oracle.backward -> oracle.sgd.  Small-integer gradients make every
    # slot's sum exact and lr = 1 makes the product exact, so the step is the correctly rounded
    # difference: bit for bit, on the region route (both record variants), the two-step route and
    # whatever the library picks; then lr = 0.01 within the float32 rounding of product and difference.
    opt = robe.options(fused_route=route, region_records=records)
    h, H = both_hashes(29 * m + Z + sign, m, d, Z, sign)
    F, B = 26, 200
    rng = np.random.default_rng(m % 1000 + d)
    ids = rng.integers(0, 3000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.3] = 11
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    g, _ = oracle.backward(H, Gi, ids, None, B, F)
    M0 = rng.standard_normal(m).astype(np.float32)
    for lr in (1.0, 0.01):
        Md = to_dev(M0)
        robe.robe_backward_sgd(h, to_dev(Gi), to_dev(ids), None, B, F, Md, lr, options=opt)
        Mo, go = M0.copy(), g.astype(np.float32)
        oracle.sgd(Mo, go, lr)
        Mg = Md.cpu().numpy()
        assert bits_equal(Mg[g == 0], M0[g == 0])
        if lr == 1.0:
            assert bits_equal(Mg, Mo)
        else:
            assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(M0) + np.abs(lr * g)) + TINY)
    # bags
    idsb, off = random_bags(rng, B * F, 3000, 6.0, long_bag=700)
    gb, _ = oracle.backward(H, Gi, idsb, off, B, F)
    Md = to_dev(M0)
    robe.robe_backward_sgd(h, to_dev(Gi), to_dev(idsb), to_dev(off), B, F, Md, 1.0, options=opt)
    Mo, go = M0.copy(), gb.astype(np.float32)
    oracle.sgd(Mo, go, 1.0)
    assert bits_equal(Md.cpu().numpy(), Mo)


@pytest.mark.parametrize("rshift", [0, 10, 15])
@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z", [(1_000_003, 128, 32), (100_003, 64, 8), (1000, 64, 32), (300_007, 128, 128), (70_001, 16, 1),
                                   (100_003, 16, 64), (250_007, 128, 512), (4099, 8, 24)])      # the last three: Z > d
def test_fused_backward_adagrad_sorted_path(m, d, Z, sign, rshift):
    # the region-sorted path: hot tokens, long bags, blocks that leave their region or wrap, one
    # region only (m = 1000), unaligned array and state
    opt = robe.options(fused_route=robe.ROUTE_REGIONS, region_shift=rshift)
    h, H = both_hashes(23 * m + Z + sign, m, d, Z, sign)
    F = 26
    B = max(8, (1 << 22) // (d * F) + 3)
    rng = np.random.default_rng(d + Z)
    ids = rng.integers(0, 4000, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.3] = 11
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    assert robe.robe_fused_workspace_bytes(h, B, F, ids.size, opt) > 8 * ids.size
    _check_fused(h, H, Gi, ids, None, B, F, m, options=opt)
    _check_fused(h, H, Gi, ids, None, B, F, m, shift=1, options=opt)
    Bb = max(4, B // 8)
    idsb, off = random_bags(rng, Bb * F, 3000, 8.0, long_bag=2500)
    _check_fused(h, H, Gi[:Bb], idsb, off, Bb, F, m, options=opt)


@pytest.mark.parametrize("sign", [0, 1])
@pytest.mark.parametrize("m,d,Z,card,rshift", [
    (1_000_003, 128, 32, 40_000, 0),     # a few hundred records per region: one round each
    (20_011, 32, 8, 1_000_000, 10),      # tens of thousands of records per region: split into classes
    (1000, 64, 32, 4000, 0),             # one region, every block overlaps hundreds of others
    (300_007, 128, 128, 3000, 13),       # blocks as long as a slice
    (300_007, 32, 128, 3000, 0),         # blocks longer than embeddings: tokens sorted by their array offset
])
def test_reproducible_mode_gives_the_same_bits_every_run(m, d, Z, card, rshift, sign):
    # No float atomics on this route and a canonical order of additions: the same call on the same
    # inputs gives the same bits, whatever order the integer atomics hand out record slots in.
    opt = robe.options(reproducible=1, region_shift=rshift)
    h, H = both_hashes(5 * m + Z + sign, m, d, Z, sign)
    F = 26
    B = max(8, (1 << 22) // (d * F) + 3)
    rng = np.random.default_rng(m + d)
    ids = rng.integers(0, card, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.2] = 7
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    M0 = rng.standard_normal(m).astype(np.float32)
    Gd, idd = to_dev(G), to_dev(ids)
    assert robe.robe_fused_workspace_bytes(h, B, F, ids.size, opt) > 8 * ids.size      # the sorted route is taken
    assert robe.robe_workspace_bytes(h, B, F, ids.size, opt) > 8 * ids.size
    runs = []
    for _ in range(4):
        Md, sd = to_dev(M0), torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward_adagrad(h, Gd, idd, None, B, F, Md, sd, 0.01, 1e-8, options=opt)
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward(h, Gd, idd, None, B, F, ga, options=opt)
        runs.append((Md.cpu().numpy(), sd.cpu().numpy(), ga.cpu().numpy()))
    for Mk, sk, gk in runs[1:]:
        assert bits_equal(Mk, runs[0][0]) and bits_equal(sk, runs[0][1]) and bits_equal(gk, runs[0][2])
    # and it is the right result
    ref, S = oracle.backward(H, G, ids, None, B, F)
    assert np.all(np.abs(runs[0][2].astype(np.float64) - ref) <= 1e-5 * S + TINY)
    # the accumulator of the fused call is the square of the very gradient the plain call returns
    g32 = runs[0][2]
    assert bits_equal(runs[0][1], g32 * g32)


def test_reproducible_mode_covers_small_problems_and_refuses_what_it_cannot_do():
    opt = robe.options(reproducible=1)
    # a handful of tokens: still the sorted route, still the right answer, bags included
    h, H = both_hashes(3, 5003, 16, 4, 1)
    rng = np.random.default_rng(0)
    B, F = 7, 5
    ids = rng.integers(0, 50, size=(B, F), dtype=np.int64)
    G = rng.standard_normal((B, F, 16)).astype(np.float32)
    assert robe.robe_workspace_bytes(h, B, F, ids.size, opt) > 0
    outs = []
    for _ in range(3):
        ga = torch.zeros(5003, dtype=torch.float32, device=DEV)
        robe.robe_backward(h, to_dev(G), to_dev(ids), None, B, F, ga, options=opt)
        outs.append(ga.cpu().numpy())
    assert bits_equal(outs[0], outs[1]) and bits_equal(outs[0], outs[2])
    ref, S = oracle.backward(H, G, ids, None, B, F)
    assert np.all(np.abs(outs[0].astype(np.float64) - ref) <= 1e-5 * S + TINY)
    flat, off = random_bags(rng, B * F, 50, 3.0)
    ga = torch.zeros(5003, dtype=torch.float32, device=DEV)
    robe.robe_backward(h, to_dev(G), to_dev(flat), to_dev(off), B, F, ga, options=opt)
    ref, S = oracle.backward(H, G, flat, off, B, F)
    assert np.all(np.abs(ga.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * S + TINY)
    Md, sd = to_dev(rng.standard_normal(5003).astype(np.float32)), torch.zeros(5003, dtype=torch.float32, device=DEV)
    robe.robe_backward_adagrad(h, to_dev(G), to_dev(flat), to_dev(off), B, F, Md, sd, 0.01, 1e-8, options=opt)
    g32 = ga.cpu().numpy()
    assert bits_equal(sd.cpu().numpy(), g32 * g32)
    # an embedding wider than the lane-group kernels take has no atomic-free route: a loud error, not a
    # silent fallback
    h2, _ = both_hashes(4, 5000, 520, 8, 0)
    ids2 = rng.integers(0, 99, size=(6, 3), dtype=np.int64)
    G2 = rng.standard_normal((6, 3, 520)).astype(np.float32)
    with pytest.raises(robe.RobeError) as ei:
        robe.robe_backward(h2, to_dev(G2), to_dev(ids2), None, 6, 3, torch.zeros(5000, dtype=torch.float32, device=DEV),
                           options=opt)
    assert ei.value.code == robe.ROBE_EINVAL and "reproducible" in str(ei.value)
    with pytest.raises(robe.RobeError):
        robe.robe_backward_adagrad(h2, to_dev(G2), to_dev(ids2), None, 6, 3, torch.zeros(5000, dtype=torch.float32, device=DEV),
                                   torch.zeros(5000, dtype=torch.float32, device=DEV), 0.01, 1e-8, options=opt)
    # without the option the same shape runs (float atomics)
    robe.robe_backward(h2, to_dev(G2), to_dev(ids2), None, 6, 3, torch.zeros(5000, dtype=torch.float32, device=DEV))
    # a block longer than the embedding is sorted by its array offset and takes the same route
    h3, H3 = both_hashes(4, 1000, 4, 16, 1)
    ids3 = rng.integers(0, 99, size=(6, 3), dtype=np.int64)
    G3 = rng.standard_normal((6, 3, 4)).astype(np.float32)
    assert robe.robe_workspace_bytes(h3, 6, 3, ids3.size, opt) > 0
    ga = torch.zeros(1000, dtype=torch.float32, device=DEV)
    robe.robe_backward(h3, to_dev(G3), to_dev(ids3), None, 6, 3, ga, options=opt)
    ref, S = oracle.backward(H3, G3, ids3, None, 6, 3)
    assert np.all(np.abs(ga.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * S + TINY)


@pytest.mark.parametrize("m,Z", [(8192 + 5, 32), (3 * 4096 + 20, 32), (2 * 32768 + 100, 64), (1024 * 5 + 31, 32)])
def test_region_route_never_leaves_a_last_region_shorter_than_a_block(m, Z):
    # With regions of 2^13 floats these arrays would end in a region of a few floats, and a block that
    # starts in the region before it would pass through it and wrap to the start of the array.  The
    # library must pick a region size without such a tail (or one region); small-integer gradients
    # make the check exact.  Many tokens, so that blocks do start in the last full region's tail.
    d, B, F = 2 * Z, 400, 26
    for sign in (0, 1):
        h, H = both_hashes(m + sign, m, d, Z, sign)
        rng = np.random.default_rng(m)
        ids = rng.integers(0, 10**6, size=(B, F), dtype=np.int64)
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        for opt in (robe.options(backward_route=robe.ROUTE_REGIONS), robe.options(reproducible=1)):
            assert robe.robe_workspace_bytes(h, B, F, ids.size, opt) > 16 * ids.size
            got, want = check_backward(h, H, Gi, ids, None, B, F, opt)
            assert np.array_equal(got, want)
        _check_fused(h, H, Gi, ids, None, B, F, m, options=robe.options(fused_route=robe.ROUTE_REGIONS))


@pytest.mark.parametrize("m,d,Z,records", [(1_000_003, 128, 32, 1), (45_000_007, 64, 64, 2), (300_007, 16, 4, 1)])
def test_region_route_when_repeated_tokens_outnumber_the_rows_of_their_sums(m, d, Z, records):
    # Every token two or three times: far more runs of repeated tokens than a lane group of the combine
    # kernel has rows for their sums (an eighth of the positions it walks).  The runs it has no row
    # for go uncombined, token by token; sums stay exact with small-integer gradients.
    B, F = 700, 26
    for sign in (0, 1):
        h, H = both_hashes(m + sign + d, m, d, Z, sign)
        rng = np.random.default_rng(d)
        ids = rng.integers(0, B * F // 3, size=(B, F), dtype=np.int64) * 1000 + np.arange(F)
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        opt = robe.options(backward_route=robe.ROUTE_REGIONS, region_records=records)
        assert robe.robe_workspace_bytes(h, B, F, ids.size, opt) > 16 * ids.size
        ref, _ = oracle.backward(H, Gi, ids, None, B, F, threads=THREADS, want_abs=False)
        for o in (opt, robe.options(reproducible=1, region_records=records)):
            ga = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward(h, to_dev(Gi), to_dev(ids), None, B, F, ga, options=o)
            nz = torch.from_numpy(np.flatnonzero(ref)).to(DEV)
            assert int(torch.count_nonzero(ga).item()) == nz.numel()
            assert np.array_equal(ga[nz].cpu().numpy().astype(np.float64), ref[nz.cpu().numpy()])


def test_reproducible_option_refuses_arrays_too_small_for_the_token_count():
    # 170,000 distinct tokens on an array of one region: far more blocks per region than the
    # canonical order handles; the call must fail, not fall back to an order that changes between runs
    m, d, Z, B, F = 8192, 32, 8, 6600, 26
    h, _ = both_hashes(5, m, d, Z, 0)
    ids = to_dev(np.arange(B * F, dtype=np.int64).reshape(B, F))
    G = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    opt = robe.options(reproducible=1)
    with pytest.raises(robe.RobeError):
        robe.robe_workspace_bytes(h, B, F, B * F, opt)
    with pytest.raises(robe.RobeError) as ei:
        robe.robe_backward(h, G, ids, None, B, F, torch.zeros(m, dtype=torch.float32, device=DEV), options=opt,
                           workspace=torch.empty(1 << 24, dtype=torch.uint8, device=DEV))
    assert ei.value.code == robe.ROBE_EINVAL and "reproducible" in str(ei.value)
    # the same problem without the option, and a smaller one with it, run
    robe.robe_backward(h, G, ids, None, B, F, torch.zeros(m, dtype=torch.float32, device=DEV))
    robe.robe_backward(h, G[:500], ids[:500], None, 500, F, torch.zeros(m, dtype=torch.float32, device=DEV), options=opt)


@pytest.mark.parametrize("m,d,Z,B,F", [(50_021, 16, 4, 9, 26), (4099, 12, 3, 5, 7), (1000, 4, 16, 6, 3), (100_003, 128, 32, 40, 26)])
def test_fused_backward_adagrad_small_problems_take_the_two_step_route(m, d, Z, B, F):
    h, H = both_hashes(m + B, m, d, Z, 1)
    rng = np.random.default_rng(B)
    ids = rng.integers(0, 50, size=(B, F), dtype=np.int64)
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    assert robe.robe_fused_workspace_bytes(h, B, F, ids.size) >= 4 * m
    _check_fused(h, H, Gi, ids, None, B, F, m)
    idsb, off = random_bags(rng, B * F, 50, 3.0, long_bag=40)
    _check_fused(h, H, Gi, idsb, off, B, F, m, shift=1)
    # nothing to do: nothing touched
    Md = torch.ones(m, device=DEV)
    sd = torch.ones(m, device=DEV)
    robe.robe_backward_adagrad(h, torch.empty((0, F, d), device=DEV), torch.empty((0, F), dtype=torch.int64, device=DEV),
                               None, 0, F, Md, sd, 0.01, 1e-8)
    assert bool((Md == 1).all()) and bool((sd == 1).all())


@pytest.mark.parametrize("m,d,Z,B,F,bags", [(50_021, 16, 4, 9, 26, False), (100_003, 128, 32, 40, 26, True)])
def test_two_step_route_twice_on_one_workspace(m, d, Z, B, F, bags):
    # The route's gradient array lives at the front of the workspace and is left holding the first
    # call's gradient; the second call must start from zeros all the same.  Exact (small-integer)
    # gradients, two Adagrad steps, against the oracle's two steps.
    h, H = both_hashes(m + 3 * B, m, d, Z, 0)
    rng = np.random.default_rng(m)
    M0 = rng.standard_normal(m).astype(np.float32)
    Md, sd = to_dev(M0), torch.zeros(m, dtype=torch.float32, device=DEV)
    Mo, so = M0.copy(), np.zeros(m, dtype=np.float32)
    n_max = 4 * B * F + 64
    need = robe.robe_fused_workspace_bytes(h, B, F, n_max)
    assert need >= 4 * m
    ws = torch.full((need,), 0x3F, dtype=torch.uint8, device=DEV)      # every float 0.747: not zeros
    for step in range(2):
        if bags:
            ids, off = random_bags(rng, B * F, 60, 3.0, long_bag=40)
            assert ids.size <= n_max
        else:
            ids, off = rng.integers(0, 60, size=(B, F), dtype=np.int64), None
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        robe.robe_backward_adagrad(h, to_dev(Gi), to_dev(ids), to_dev(off), B, F, Md, sd, 0.01, 1e-8, workspace=ws)
        g, _ = oracle.backward(H, Gi, ids, off, B, F)
        assert np.array_equal(g, np.round(g))
        oracle.adagrad(Mo, so, g.astype(np.float32), 0.01, 1e-8)
        Mg, sg = Md.cpu().numpy(), sd.cpu().numpy()
        assert bits_equal(sg, so), step                     # the accumulator is exact: sums of squares of small integers
        assert np.all(np.abs(Mg.astype(np.float64) - Mo) <= 1e-6 * (np.abs(Mo) + 0.02) + TINY), step


def _bag_forward_ok(h, H, M, idsb, off, B, F, options):
    outb = robe.robe_forward(h, to_dev(M), to_dev(idsb), to_dev(off), B, F, options=options).cpu().numpy()
    want = oracle.forward(H, M, idsb, off, B, F, threads=THREADS)
    H_abs = oracle.Hash(H.m, H.d, H.Z, 0, H.P, H.coef)
    S = oracle.forward(H_abs, np.abs(M), idsb, off, B, F, threads=THREADS).astype(np.float64)
    err = np.abs(outb.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= 1e-5 * S + TINY), float((err / (S + TINY)).max())


@pytest.mark.parametrize("fields", [dict(fwd_elems=4), dict(fwd_elems=2), dict(fwd_elems=1),
                                    dict(fwd_elems=4, fwd_strided=1), dict(fwd_elems=2, fwd_strided=1), dict(fwd_elems=-1),
                                    dict(bwd_elems=4), dict(bwd_elems=2), dict(bwd_elems=4, bwd_strided=1),
                                    dict(bwd_elems=2, bwd_strided=1), dict(bwd_elems=-1), dict(tile_lookups=64),
                                    dict(tile_lookups=8), dict(row_order=robe.ROWS_BY_TABLE_ALWAYS),
                                    dict(row_order=robe.ROWS_MEMORY)])
def test_every_lane_layout_gives_the_same_result(fields):
    # d = 64 makes every (elements per lane, layout) legal
    opt = robe.options(**fields)
    m, d, Z, B, F = 60_013, 64, 16, 41, 26
    for sign in (0, 1):
        h, H = both_hashes(99, m, d, Z, sign)
        rng = np.random.default_rng(5)
        ids = rng.integers(0, 3000, size=(B, F), dtype=np.int64)
        M = workloads.make_array(m, 9)
        out = robe.robe_forward(h, to_dev(M), to_dev(ids), None, B, F, options=opt)
        assert bits_equal(out.cpu().numpy(), oracle.forward(H, M, ids, None, B, F, threads=THREADS))
        idsb, off = random_bags(rng, B * F, 3000, 7.0, long_bag=100)
        _bag_forward_ok(h, H, M, idsb, off, B, F, opt)
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        for (i_, o_) in ((ids, None), (idsb, off)):
            ga = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward(h, to_dev(Gi), to_dev(i_), to_dev(o_), B, F, ga, options=opt)
            want, _ = oracle.backward(H, Gi, i_, o_, B, F)
            assert np.array_equal(ga.cpu().numpy().astype(np.float64), want)


def test_options_that_do_not_fit_are_errors_not_silent_defaults():
    h, _ = both_hashes(1, 10_007, 48, 16, 0)
    M = torch.zeros(10_007, dtype=torch.float32, device=DEV)
    ids = torch.zeros((4, 3), dtype=torch.int64, device=DEV)
    for fields in (dict(fwd_elems=5), dict(fwd_elems=4), dict(fwd_elems=3), dict(tile_lookups=3), dict(row_order=9),
                   dict(region_shift=9), dict(key_bits=40), dict(backward_route=7), dict(reproducible=2)):
        with pytest.raises(robe.RobeError) as ei:      # 48 / 4 = 12 lanes, 3 consecutive: neither exists
            robe.robe_forward(h, M, ids, None, 4, 3, options=robe.options(**fields))
        assert ei.value.code == robe.ROBE_EINVAL, fields
    robe.robe_forward(h, M, ids, None, 4, 3, options=robe.options(fwd_elems=3, fwd_strided=1))


@pytest.mark.parametrize("B,F", [(1, 2), (3, 26), (37, 26), (64, 5), (1000, 3), (5, 64), (129, 1)])
@pytest.mark.parametrize("xcd", [robe.ROWS_MEMORY, robe.ROWS_BY_TABLE_ALWAYS])
def test_row_walk_orders_cover_every_row_once(B, F, xcd):
    # rows walked in memory order or table by table (an eighth of that order per XCD): same results,
    # for batches smaller than a tile, tables that end inside a tile, and grids padded to 8 XCDs
    opt = robe.options(row_order=xcd, backward_route=robe.ROUTE_DIRECT)
    for (m, d, Z) in [(50_021, 128, 32), (9_973, 16, 4), (30_011, 128, 1)]:
        h, H = both_hashes(B * 131 + F, m, d, Z, 1)
        rng = np.random.default_rng(B + F)
        ids = rng.integers(0, 2000, size=(B, F), dtype=np.int64)
        M = workloads.make_array(m, 2)
        out = robe.robe_forward(h, to_dev(M), to_dev(ids), None, B, F, options=opt)
        assert bits_equal(out.cpu().numpy(), oracle.forward(H, M, ids, None, B, F, threads=THREADS))
        idsb, off = random_bags(rng, B * F, 2000, 4.0, long_bag=70)
        _bag_forward_ok(h, H, M, idsb, off, B, F, opt)
        Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
        for (i_, o_) in ((ids, None), (idsb, off)):
            ga = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward(h, to_dev(Gi), to_dev(i_), to_dev(o_), B, F, ga, options=opt)
            want, _ = oracle.backward(H, Gi, i_, o_, B, F)
            assert np.array_equal(ga.cpu().numpy().astype(np.float64), want)


def test_empty_problems_and_all_empty_bags():
    h, H = both_hashes(8, 10_007, 16, 4, 1)
    M = to_dev(workloads.make_array(10_007, 0))
    F = 3
    # batch 0: nothing launched, nothing touched
    out0 = robe.robe_forward(h, M, torch.empty((0, F), dtype=torch.int64, device=DEV), None, 0, F)
    assert out0.shape == (0, F, 16)
    ga = torch.full((10_007,), 2.0, dtype=torch.float32, device=DEV)
    robe.robe_backward(h, torch.empty((0, F, 16), device=DEV), torch.empty((0, F), dtype=torch.int64, device=DEV),
                       None, 0, F, ga)
    assert bool((ga == 2.0).all())
    # rows exist but every bag is empty: zeros out, gradient array untouched, no index buffer needed
    B = 5
    off = torch.zeros(B * F + 1, dtype=torch.int64, device=DEV)
    none = torch.empty(0, dtype=torch.int64, device=DEV)
    out = robe.robe_forward(h, M, none, off, B, F)
    assert not out.cpu().numpy().any() and not np.signbit(out.cpu().numpy()).any()
    robe.robe_backward(h, torch.ones((B, F, 16), device=DEV), none, off, B, F, ga)
    assert bool((ga == 2.0).all())
    rc = robe.lib().robe_forward(ctypes.byref(h), M.data_ptr(), None, off.data_ptr(), 0, B, F, out.data_ptr(), None, None)
    assert rc == robe.ROBE_OK


def test_malformed_csr_is_clamped_not_followed():
    # every bag's bounds are clamped to [0, n_indices] on their own and a negative length becomes empty
    h, H = both_hashes(1, 10_007, 16, 4, 0)
    B, F = 2, 2
    ids = np.arange(10, dtype=np.int64)
    bad = np.array([0, 3, 50, 7, 10], dtype=np.int64)           # bags: [0,3) [3,50) [50,7) [7,10)
    same_ids = np.concatenate([ids[0:3], ids[3:10], ids[7:10]])  # ...which clamp to [0,3) [3,10) [] [7,10)
    same_off = np.array([0, 3, 10, 10, 13], dtype=np.int64)
    M = workloads.make_array(10_007, 0)
    out = robe.robe_forward(h, to_dev(M), to_dev(ids), to_dev(bad), B, F).cpu().numpy()
    want = oracle.forward(H, M, same_ids, same_off, B, F)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-7)


def test_runs_on_a_side_stream_and_reports_bad_sizes():
    h, H = both_hashes(4, 20_011, 16, 4, 1)
    B, F = 16, 26
    ids = np.random.default_rng(2).integers(0, 1000, size=(B, F), dtype=np.int64)
    M = workloads.make_array(20_011, 0)
    Md, idd = to_dev(M), to_dev(ids)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out = robe.robe_forward(h, Md, idd, None, B, F)
    s.synchronize()
    assert bits_equal(out.cpu().numpy(), oracle.forward(H, M, ids, None, B, F))
    rc = robe.lib().robe_forward(ctypes.byref(h), Md.data_ptr(), idd.data_ptr(), None,
                                 B * F + 1, B, F, out.data_ptr(), None, None)
    assert rc == robe.ROBE_EINVAL and b"n_indices" in robe.lib().robe_last_error()


@pytest.mark.parametrize("m,modes", [(2**30, ("direct", "dedup", "regions")), (2**31 - 1, ("direct", "dedup"))])
def test_backward_on_the_largest_arrays(m, modes):
    # 2^30 slots is the largest array the region-sorted route takes (32768 regions of 2^15 floats),
    # 2^31 - 1 the largest array at all; small-integer gradients make every route exact
    d, Z, B, F = 128, 32, 2048, 26
    rng = np.random.default_rng(m % 1000)
    h, H = both_hashes(99, m, d, Z, 1)
    sizes = rng.poisson(4.0, size=B * F).astype(np.int64)
    off = np.zeros(B * F + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    ids = rng.integers(0, 10**5, size=int(off[-1]), dtype=np.int64)
    ids[rng.random(ids.size) < 0.2] = 5
    G = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    ref, _ = oracle.backward(H, G, ids, off, B, F, threads=THREADS, want_abs=False)
    nz = np.flatnonzero(ref)
    Gd, idd, offd = to_dev(G), to_dev(ids), to_dev(off)
    for mode in modes:
        opt = robe.options(backward_route=ROUTES[mode], fused_route=robe.ROUTE_REGIONS)
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward(h, Gd, idd, offd, B, F, ga, options=opt)
        assert int(torch.count_nonzero(ga).item()) == nz.size, mode
        assert np.array_equal(ga[torch.from_numpy(nz).to(DEV)].cpu().numpy().astype(np.float64), ref[nz]), mode
        del ga
        if mode == "regions":
            Md = torch.zeros(m, dtype=torch.float32, device=DEV)
            sd = torch.zeros(m, dtype=torch.float32, device=DEV)
            robe.robe_backward_adagrad(h, Gd, idd, offd, B, F, Md, sd, 0.01, 1e-8, options=opt)
            assert int(torch.count_nonzero(sd).item()) == nz.size
            got_s = sd[torch.from_numpy(nz).to(DEV)].cpu().numpy()
            assert np.array_equal(got_s, ref[nz].astype(np.float32) ** 2)
            del Md, sd
    torch.cuda.empty_cache()
