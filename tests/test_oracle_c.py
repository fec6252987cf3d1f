"""The plain-C reference tier must reproduce the pure-Python tier exactly (which is itself pinned by
brute force / CRT / closed forms) on every entry point, including shrunken replicas of the large
workload shapes (same L, K, dnum, ragged last digit) at a small ring degree."""

import random

import numpy as np
import pytest

import ks_inputs
from oracle import ckks_ref as R


def _setup(c_tier, logN, L, K, dnum):
    pl = R.ntt_primes(logN, L + K)
    pr = R.Params(logN, pl[K:], pl[:K], dnum)
    co = c_tier.COracle(logN, pr.q, pr.p, dnum, pr.psi)
    return pr, co


def _rand(rng, pr, ids):
    return [[rng.randrange(pr.moduli[m]) for _ in range(pr.N)] for m in ids]


def _np(x):
    return np.asarray(x, dtype=np.uint64)


def _rand_key(rng, pr):
    ids = list(range(pr.L + pr.K))
    return [[_rand(rng, pr, ids), _rand(rng, pr, ids)] for _ in range(len(pr.digits(pr.L)))]


@pytest.mark.parametrize("logN", [4, 9, 12])
def test_c_ntt_matches_python(c_oracle_lib, logN):
    pr, co = _setup(c_oracle_lib, logN, 3, 2, 1)
    rng = random.Random(logN)
    ids = [0, 2, 4, 3]
    x = _rand(rng, pr, ids)
    fwd = co.ntt_fwd(_np(x)[None], ids)[0]
    want = [R.ntt(x[i], pr.moduli[m], pr.psi[m]) for i, m in enumerate(ids)]
    assert fwd.tolist() == want
    back = co.ntt_inv(fwd[None], ids)[0]
    assert back.tolist() == x
    assert co.ntt_inv(_np(x)[None], ids)[0].tolist() == [R.intt(x[i], pr.moduli[m], pr.psi[m]) for i, m in enumerate(ids)]


def test_c_bconv_matches_python(c_oracle_lib):
    pr, co = _setup(c_oracle_lib, 6, 6, 3, 2)
    rng = random.Random(2)
    src_ids, dst_ids = [0, 1, 2], [3, 4, 5, 6, 7, 8]
    x = [_rand(rng, pr, src_ids) for _ in range(2)]
    got = co.bconv(_np(x), src_ids, dst_ids)
    for b in range(2):
        want = R.bconv_fast(x[b], [pr.moduli[m] for m in src_ids], [pr.moduli[m] for m in dst_ids])
        assert got[b].tolist() == want


@pytest.mark.parametrize("logN,L,K,dnum,ell", [(5, 4, 2, 2, 4), (6, 5, 2, 3, 5), (6, 6, 3, 2, 4),
                                               (8, 24, 8, 3, 24), (8, 35, 12, 3, 35)])
def test_c_keyswitch_matches_python(c_oracle_lib, logN, L, K, dnum, ell):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(L)
    evk = _rand_key(rng, pr)
    d = _rand(rng, pr, range(ell))
    got = co.keyswitch(_np(d)[None], _np(evk), ell)[0]
    o0, o1 = R.keyswitch(pr, d, evk, ell)
    assert got[0].tolist() == o0 and got[1].tolist() == o1


def test_c_keyswitch_cfg1_matches_python(c_oracle_lib):
    cfg = ks_inputs.CONFIGS[1]
    q, p = ks_inputs.moduli(cfg)
    pr = R.Params(cfg["logN"], q, p, cfg["dnum"])
    co = c_oracle_lib.COracle(cfg["logN"], q, p, cfg["dnum"], pr.psi)
    evk_t = ks_inputs.uniform_residues(cfg["seed"], 2, (cfg["dnum"], 2), pr.moduli, pr.N)
    d_t = ks_inputs.uniform_residues(cfg["seed"], 1, (1,), pr.q, pr.N)
    got = co.keyswitch(ks_inputs.as_u64(d_t), ks_inputs.as_u64(evk_t))[0]
    o0, o1 = R.keyswitch(pr, d_t[0].tolist(), evk_t.tolist())
    assert got[0].tolist() == o0 and got[1].tolist() == o1


@pytest.mark.parametrize("logN,L,K,dnum", [(5, 4, 2, 2), (7, 24, 8, 3)])
def test_c_rotate_hoisted_matches_python(c_oracle_lib, logN, L, K, dnum):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(3)
    galois = ks_inputs.galois_elements(logN, 3)
    keys = [_rand_key(rng, pr) for _ in galois]
    cts = [(_rand(rng, pr, range(L)), _rand(rng, pr, range(L))) for _ in range(2)]
    got = co.rotate_hoisted(_np([[c0, c1] for c0, c1 in cts]), galois, [_np(k) for k in keys])
    for b, ct in enumerate(cts):
        want = R.rotate_hoisted(pr, ct, galois, keys)
        for r, (o0, o1) in enumerate(want):
            assert got[b, r, 0].tolist() == o0 and got[b, r, 1].tolist() == o1


@pytest.mark.parametrize("logN,L,K,dnum,ell", [(5, 4, 2, 2, 4), (6, 24, 8, 3, 24), (6, 6, 2, 3, 5)])
def test_c_rotate_mac_matches_python(c_oracle_lib, logN, L, K, dnum, ell):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(7)
    galois = ks_inputs.galois_elements(logN, 3)
    keys = [_rand_key(rng, pr) for _ in galois]
    pts = [_rand(rng, pr, range(L + K)) for _ in galois]
    cts = [(_rand(rng, pr, range(ell)), _rand(rng, pr, range(ell))) for _ in range(2)]
    got = co.rotate_mac_hoisted(_np([[c0, c1] for c0, c1 in cts]), galois, [_np(k) for k in keys], [_np(w) for w in pts], ell)
    for b, ct in enumerate(cts):
        o0, o1 = R.rotate_mac_hoisted(pr, ct, galois, keys, pts, ell)
        assert got[b, 0].tolist() == o0 and got[b, 1].tolist() == o1


@pytest.mark.parametrize("logN,L,K,dnum,ell", [(5, 4, 2, 2, 4), (6, 6, 2, 3, 5)])
def test_c_bsgs_matches_python(c_oracle_lib, logN, L, K, dnum, ell):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(8)
    gal = ks_inputs.galois_elements(logN, 3)
    baby, giant = [1, gal[0], gal[1]], [1, gal[2]]
    bkeys = [None] + [_rand_key(rng, pr) for _ in baby[1:]]
    gkeys = [None] + [_rand_key(rng, pr) for _ in giant[1:]]
    pts = [[_rand(rng, pr, range(L + K)) for _ in baby] for _ in giant]
    pts[1][0] = None                                             # a unit plaintext
    cts = [(_rand(rng, pr, range(ell)), _rand(rng, pr, range(ell))) for _ in range(2)]
    npk = lambda k: None if k is None else _np(k)
    got = co.bsgs_linear_transform(_np([[c0, c1] for c0, c1 in cts]), baby, [npk(k) for k in bkeys], giant, [npk(k) for k in gkeys],
                                   [[npk(w) for w in row] for row in pts], ell)
    for b, ct in enumerate(cts):
        o0, o1 = R.bsgs_linear_transform(pr, ct, baby, bkeys, giant, gkeys, pts, ell)
        assert got[b, 0].tolist() == o0 and got[b, 1].tolist() == o1
    # the identity element and the unit plaintext in the single-level entry point
    got = co.rotate_mac_hoisted(_np([list(cts[0])]), baby, [npk(k) for k in bkeys], [npk(w) for w in pts[1]], ell)[0]
    o0, o1 = R.rotate_mac_hoisted(pr, cts[0], baby, bkeys, pts[1], ell)
    assert got[0].tolist() == o0 and got[1].tolist() == o1


@pytest.mark.parametrize("logN,L,K,dnum", [(5, 4, 2, 2), (7, 35, 12, 3)])
def test_c_hmult_matches_python(c_oracle_lib, logN, L, K, dnum):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(4)
    rlk = _rand_key(rng, pr)
    cta = (_rand(rng, pr, range(L)), _rand(rng, pr, range(L)))
    ctb = (_rand(rng, pr, range(L)), _rand(rng, pr, range(L)))
    got = co.hmult_relin_rescale(_np([list(cta)]), _np([list(ctb)]), _np(rlk))[0]
    o0, o1 = R.hmult_relin_rescale(pr, cta, ctb, rlk)
    assert got[0].tolist() == o0 and got[1].tolist() == o1


@pytest.mark.parametrize("logN,L,K,dnum,ell", [(5, 4, 2, 2, 4), (7, 35, 12, 3, 35), (6, 6, 2, 3, 4)])
def test_c_hmult_merged_matches_python(c_oracle_lib, logN, L, K, dnum, ell):
    pr, co = _setup(c_oracle_lib, logN, L, K, dnum)
    rng = random.Random(6)
    rlk = _rand_key(rng, pr)
    cta = (_rand(rng, pr, range(ell)), _rand(rng, pr, range(ell)))
    ctb = (_rand(rng, pr, range(ell)), _rand(rng, pr, range(ell)))
    got = co.hmult_relin_rescale_merged(_np([list(cta)]), _np([list(ctb)]), _np(rlk), ell)[0]
    o0, o1 = R.hmult_relin_rescale_merged(pr, cta, ctb, rlk, ell)
    assert got[0].tolist() == o0 and got[1].tolist() == o1


def test_input_generator_is_counter_based():
    """Any slab regenerated alone equals the same slab of the whole tensor; residues are in range."""
    mods = R.ntt_primes(12, 3)
    whole = ks_inputs.uniform_residues(5, 9, (2, 3), mods, 64)
    assert whole.shape == (2, 3, 3, 64)
    assert (whole[1, 2] == ks_inputs.uniform_slab(5, 9, 5, mods, 64)).all()
    m = np.asarray(mods, dtype=np.int64).reshape(1, 1, 3, 1)
    w = whole.numpy()
    assert (w >= 0).all() and (w < m).all()
    # first element by hand: SplitMix64 finaliser of the key, top 36 bits, reduced
    mask = (1 << 64) - 1
    z = (5 * 0x9E3779B97F4A7C15 + 9 * 0xD1B54A32D192ED03) & mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    z ^= z >> 31
    assert int(whole[0, 0, 0, 0]) == (z >> 28) % mods[0]


def test_checksum_sees_value_and_position():
    import torch
    from checksum import checksum
    x = torch.arange(1000, dtype=torch.int64) * 977 % 68718428161
    base = checksum(x)
    y = x.clone(); y[123] += 1
    assert checksum(y) != base
    z = x.clone(); z[[5, 900]] = z[[900, 5]]
    assert checksum(z) != base
    assert checksum(x.view(10, 100)) == base           # shape does not matter, order does


def test_stored_fullsize_checksums_come_from_the_reference(c_oracle_lib):
    """Spot check of tests/golden/fullsize_checksums.txt: one multiplication of configuration 5 recomputed here."""
    import os
    import torch
    from checksum import checksum
    path = os.path.join(os.path.dirname(__file__), "golden", "fullsize_checksums.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert sum(r[0] == "cfg3_rotate" for r in rows) == 64 * 16
    assert sum(r[0] == "cfg5_hmult" for r in rows) == 256 and sum(r[0] == "cfg5_hmult_merged" for r in rows) == 256
    table = {(r[0], int(r[1]), int(r[2])): (int(r[3], 16), int(r[4], 16)) for r in rows}
    cfg = ks_inputs.CONFIGS[5]
    q, p = ks_inputs.moduli(cfg)
    N, L, seed, b = 1 << cfg["logN"], cfg["L"], cfg["seed"], 201
    co = c_oracle_lib.COracle(cfg["logN"], q, p, cfg["dnum"], [R.minimal_psi(m, cfg["logN"]) for m in q + p])
    u64 = lambda t: t.numpy().view(np.uint64)
    rlk = u64(ks_inputs.uniform_residues(seed, 3, (cfg["dnum"], 2), q + p, N))
    cta = np.stack([u64(ks_inputs.uniform_slab(seed, 1, 2 * b + c, q, N)) for c in range(2)])[None]
    ctb = np.stack([u64(ks_inputs.uniform_slab(seed, 2, 2 * b + c, q, N)) for c in range(2)])[None]
    out = co.hmult_relin_rescale_merged(cta, ctb, rlk, L)[0]
    assert checksum(torch.from_numpy(np.ascontiguousarray(out).view(np.int64))) == table[("cfg5_hmult_merged", b, 0)]
