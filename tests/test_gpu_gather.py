"""The region route whose reduce kernel finds its blocks in the sorted token list (no record
kernels): parity with the oracle on arrays large enough for its range table, slot by slot.
Small-integer gradients make every float32 sum exact, so the comparison is bit for bit; cases cover
a region that ends the array short of a block, blocks that wrap to slot 0, tokens repeated thousands
of times, bags, a coarse sort key (wide directory buckets), the sign hash, the fused Adagrad write-back
and the reproducible option."""
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


def hashes(seed, m, d, Z, sign):
    h = robe.robe_init_hash(seed, m, d, Z, sign)
    H = oracle.init_hash(seed, m, d, Z, sign)
    assert tuple(h.coef) == H.coef
    return h, H


def tokens_near_the_array_end(H, F, want, rng):
    """Ids whose first block starts within a few slots of the end of the array (found by trying ids
    against the oracle's offsets): their blocks wrap to slot 0 or pass through a short last region."""
    found = []
    while len(found) < want:
        ids = rng.integers(0, 2**40, size=200_000 // F * F, dtype=np.int64)
        off = oracle.offsets(H, ids, F)[:, 0]
        hit = np.flatnonzero(off >= H.m - 40)
        found.extend((int(ids[k]), int(k % F)) for k in hit)
    return found[:want]


# (m, d, Z, sign, key_bits, region_shift).  The range table holds (d/Z) * ((2^31 - 2) / m + 3) entries:
# at most 120 (56 with the sign), hence arrays of tens of millions of slots.
CASES = [
    (25_000_000 + 5, 32, 32, 0, 0, 0),         # 88 entries; the last region holds 6925 floats
    (45_000_007, 32, 32, 1, 0, 0),             # 50 entries, sign on
    (3 * 8192 * 1024 + 5, 32, 32, 0, 0, 0),    # the array ends in a region of 5 floats: blocks pass through it to slot 0
    (2**26 + 3, 64, 32, 0, 0, 13),             # two chunks per embedding, 68 entries
    (2**27 + 3, 128, 64, 1, 16, 0),            # a coarse sort key: distinct tokens share keys, wide directory buckets
    (40_000_003, 32, 16, 0, 8, 14),            # 8 key bits: 256 directory buckets; regions of 2^14 floats; 112 entries
    (250_000_000, 128, 32, 1, 0, 0),           # the headline shape, sign on
    (2**26 + 3, 16, 64, 0, 0, 0),              # blocks larger than embeddings: keys are array offsets below 2^27
    (45_000_007, 32, 128, 1, 0, 0),            # the same with the sign, keys below 2^26
    (70_000_001, 8, 24, 0, 12, 0),             # three embeddings per block, 12 key bits of 27
]


@pytest.mark.parametrize("m,d,Z,sign,key_bits,rshift", CASES)
def test_gather_route_matches_the_oracle(m, d, Z, sign, key_bits, rshift):
    h, H = hashes(m + d + sign, m, d, Z, sign)
    F, B = 26, 600
    rng = np.random.default_rng(m % 9973 + Z)
    ids = rng.integers(0, 10**6, size=(B, F), dtype=np.int64)
    ids[rng.random((B, F)) < 0.25] = 11                       # one token thousands of times: many runs of one key
    for k, (x, f) in enumerate(tokens_near_the_array_end(H, F, 64, rng)):
        ids[k * 7 % B, f] = x
    Gi = rng.integers(-3, 4, size=(B, F, d)).astype(np.float32)
    base = dict(region_records=2, region_shift=rshift, key_bits=key_bits)
    opt = robe.options(backward_route=robe.ROUTE_REGIONS, **base)
    records = robe.options(backward_route=robe.ROUTE_REGIONS, region_records=1, region_shift=rshift, key_bits=key_bits)
    # the gather variant is what runs: it needs no record storage, so its workspace is the smaller one
    assert 0 < robe.robe_workspace_bytes(h, B, F, ids.size, opt) < robe.robe_workspace_bytes(h, B, F, ids.size, records)
    ref, _ = oracle.backward(H, Gi, ids, None, B, F, threads=8)
    nz = np.flatnonzero(ref)
    nzd = torch.from_numpy(nz).to(DEV)
    Gd, idd = dev(Gi), dev(ids)

    def check(ga, what):
        assert int(torch.count_nonzero(ga).item()) == nz.size, what
        assert np.array_equal(ga[nzd].cpu().numpy().astype(np.float64), ref[nz]), what

    ga = torch.zeros(m, dtype=torch.float32, device=DEV)
    robe.robe_backward(h, Gd, idd, None, B, F, ga, options=opt)
    check(ga, "single-hot")
    # bags over the same ids: every token receives its bag's row
    sizes = rng.poisson(2.0, size=B * F).astype(np.int64)
    sizes[5] = 3000
    off = np.zeros(B * F + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    flat = rng.integers(0, 3000, size=int(off[-1]), dtype=np.int64)
    refb, _ = oracle.backward(H, Gi, flat, off, B, F, threads=8)
    ga.zero_()
    robe.robe_backward(h, Gd, dev(flat), dev(off), B, F, ga, options=opt)
    nzb = np.flatnonzero(refb)
    assert int(torch.count_nonzero(ga).item()) == nzb.size
    assert np.array_equal(ga[torch.from_numpy(nzb).to(DEV)].cpu().numpy().astype(np.float64), refb[nzb])
    # reproducible option on the same variant: same exact sums
    ga.zero_()
    robe.robe_backward(h, Gd, idd, None, B, F, ga, options=robe.options(reproducible=1, **base))
    check(ga, "reproducible")
    # fused Adagrad from zero state: the accumulator is the square of the exact gradient, untouched slots stay
    Md = torch.full((m,), 0.5, dtype=torch.float32, device=DEV)
    sd = torch.zeros(m, dtype=torch.float32, device=DEV)
    robe.robe_backward_adagrad(h, Gd, idd, None, B, F, Md, sd, 0.01, 1e-8,
                               options=robe.options(fused_route=robe.ROUTE_REGIONS, **base))
    assert int(torch.count_nonzero(sd).item()) == nz.size
    assert np.array_equal(sd[nzd].cpu().numpy(), ref[nz].astype(np.float32) ** 2)
    assert int(torch.count_nonzero(Md != 0.5).item()) == nz.size
    g = ref[nz].astype(np.float32)
    want_M = np.float32(0.5) - (np.float32(0.01) * g) / (np.abs(g) + np.float32(1e-8))
    assert np.all(np.abs(Md[nzd].cpu().numpy().astype(np.float64) - want_M) <= 1e-6)


@pytest.mark.parametrize("sign", [0, 1])
def test_gather_route_is_reproducible_with_real_gradients(sign):
    # real-valued gradients and enough tokens per region for rounding to depend on the order: four
    # runs of the reproducible option give the same bits, and agree with the oracle to the usual bar
    m, d, Z = 45_000_017, 32, 32
    h, H = hashes(3 + sign, m, d, Z, sign)
    F, B = 26, 3000
    rng = np.random.default_rng(sign)
    ids = rng.integers(0, 2000, size=(B, F), dtype=np.int64)            # 52,000 distinct tokens at most: every slot many times
    G = rng.standard_normal((B, F, d)).astype(np.float32)
    opt = robe.options(reproducible=1, region_records=2)
    Gd, idd = dev(G), dev(ids)
    runs = []
    for _ in range(4):
        ga = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward(h, Gd, idd, None, B, F, ga, options=opt)
        Md = torch.zeros(m, dtype=torch.float32, device=DEV)
        sd = torch.zeros(m, dtype=torch.float32, device=DEV)
        robe.robe_backward_adagrad(h, Gd, idd, None, B, F, Md, sd, 0.01, 1e-8, options=opt)
        runs.append((ga.cpu().numpy(), sd.cpu().numpy(), Md.cpu().numpy()))
        del ga, Md, sd
    for gk, sk, Mk in runs[1:]:
        assert bits_equal(gk, runs[0][0]) and bits_equal(sk, runs[0][1]) and bits_equal(Mk, runs[0][2])
    ref, S = oracle.backward(H, G, ids, None, B, F, threads=8)
    assert np.all(np.abs(runs[0][0].astype(np.float64) - ref) <= 1e-5 * S + TINY)
    assert bits_equal(runs[0][1], runs[0][0] * runs[0][0])
