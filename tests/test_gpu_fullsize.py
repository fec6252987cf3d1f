"""GPU parity at the full workload sizes, in the launch configuration the benchmark uses.

The outputs are too large for the CPU reference to recompute entirely (24 GiB of hoisted rotations, 256
multiplications at N = 2^16), so the reference recomputes sampled batch items / rotations one by one and
those must match bit-exactly; properties that hold for the whole tensor (exact round trip, residues in
range) are checked everywhere."""

import os

import numpy as np
import pytest
import torch

import ks_inputs
import paper_2512_11269_amd as K
from checksum import checksum
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu


def _golden_checksums():
    """(workload, item, sub-item) -> (c1, c2): checksums of the CPU reference's full-size outputs, computed ahead of time by
    tests/golden/make_fullsize_checksums.py (reference and seeded inputs only)."""
    table = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "fullsize_checksums.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, a, b, c1, c2 = line.split()
            table[(name, int(a), int(b))] = (int(c1, 16), int(c2, 16))
    return table


def _assert_all_items_match(name, items, table):
    """items: iterable of ((item, sub-item), tensor).  Every one must reproduce the reference's checksums."""
    bad = [(key, got) for key, t in items if (got := checksum(t)) != table[(name,) + key]]
    assert not bad, f"{len(bad)} outputs differ from the reference, first {bad[0][0]}"


def _in_range(t, mods):
    m = torch.tensor(mods, dtype=torch.int64, device=t.device).view(len(mods), 1)
    return bool(((t >= 0) & (t < m)).all())


def test_cfg4_batched_ntt_full_size():
    cfg = ks_inputs.CONFIGS[4]
    st = Setup(cfg["logN"], cfg["L"], 0, 1)
    ids = list(range(cfg["L"]))
    x = st.uniform(cfg["seed"], 1, (cfg["batch"],), ids)
    y = x.clone()
    K.ntt_fwd(st.ctx, y, ids)
    assert _in_range(y, st.q)
    # two whole polynomials (every one of the 60 moduli, so a wrong root or table of any modulus shows) and a few more
    # sampled limbs against the reference; the round trip covers the rest
    for b in (0, cfg["batch"] - 1):
        assert_equal(y[b], st.ref.ntt_fwd(host(x[b])[None], ids)[0])
    rng = np.random.RandomState(4)
    for _ in range(6):
        b, i = int(rng.randint(cfg["batch"])), int(rng.randint(cfg["L"]))
        want = st.ref.ntt_fwd(host(x[b, i])[None, None], [i])
        assert_equal(y[b, i], want[0, 0])
    z = x[3].clone()
    K.ntt_inv(st.ctx, z, ids)                       # the inverse alone on a whole polynomial, not only as a round trip
    assert_equal(z, st.ref.ntt_inv(host(x[3])[None], ids)[0])
    K.ntt_inv(st.ctx, y, ids)
    assert torch.equal(y, x)


def test_cfg3_hoisted_rotations_full_size():
    cfg = ks_inputs.CONFIGS[3]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"])
    ell, B, n_rot, seed = cfg["L"], cfg["batch"], cfg["n_rot"], cfg["seed"]
    ct = st.uniform(seed, 1, (B, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (cfg["dnum"], 2), list(range(ell + cfg["K"]))) for r in range(n_rot)]
    galois = ks_inputs.galois_elements(cfg["logN"], n_rot)
    out = torch.empty((B, n_rot, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_hoisted(st.ctx, ct, ell, galois, keys, out, workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, B, n_rot))
    torch.cuda.synchronize()
    for b, r in [(0, 0), (17, 5), (63, 15), (16, 9)]:      # first, last, chunk boundary, middle
        want = st.ref.rotate_hoisted(host(ct[b])[None], [galois[r]], [host(keys[r])], ell)
        assert_equal(out[b, r], want[0, 0])
    for b in (1, 40):
        assert _in_range(out[b].reshape(-1, ell, st.N), st.q)
    # every one of the 1024 rotated ciphertexts (24 GiB) against the reference's checksums
    _assert_all_items_match("cfg3_rotate", (((b, r), out[b, r]) for b in range(B) for r in range(n_rot)), _golden_checksums())


def test_cfg5_hmult_full_size():
    cfg = ks_inputs.CONFIGS[5]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"])
    ell, B, seed = cfg["L"], cfg["batch"], cfg["seed"]
    cta = st.uniform(seed, 1, (B, 2), list(range(ell)))
    ctb = st.uniform(seed, 2, (B, 2), list(range(ell)))
    rlk = st.uniform(seed, 3, (cfg["dnum"], 2), list(range(ell + cfg["K"])))
    out = torch.empty((B, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
    K.hmult_relin_rescale(st.ctx, cta, ctb, ell, rlk, out, workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, B))
    torch.cuda.synchronize()
    for b in (0, 15, 16, 255):
        want = st.ref.hmult_relin_rescale(host(cta[b])[None], host(ctb[b])[None], host(rlk), ell)
        assert_equal(out[b], want[0])
    assert _in_range(out[100].reshape(-1, ell - 1, st.N), st.q[:ell - 1])
    _assert_all_items_match("cfg5_hmult", (((b, 0), out[b]) for b in range(B)), _golden_checksums())


def test_cfg5_hmult_merged_full_size():
    cfg = ks_inputs.CONFIGS[5]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"])
    ell, B, seed = cfg["L"], cfg["batch"], cfg["seed"]
    cta = st.uniform(seed, 1, (B, 2), list(range(ell)))
    ctb = st.uniform(seed, 2, (B, 2), list(range(ell)))
    rlk = st.uniform(seed, 3, (cfg["dnum"], 2), list(range(ell + cfg["K"])))
    out = torch.empty((B, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
    K.hmult_relin_rescale_merged(st.ctx, cta, ctb, ell, rlk, out, workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, B))
    torch.cuda.synchronize()
    for b in (0, 16, 255):
        want = st.ref.hmult_relin_rescale_merged(host(cta[b])[None], host(ctb[b])[None], host(rlk), ell)
        assert_equal(out[b], want[0])
    assert _in_range(out[77].reshape(-1, ell - 1, st.N), st.q[:ell - 1])
    _assert_all_items_match("cfg5_hmult_merged", (((b, 0), out[b]) for b in range(B)), _golden_checksums())


def test_cfg3_rotate_mac_full_size():
    """Configuration 3's shape through the double-hoisted entry point: 64 ciphertexts, 16 rotations summed."""
    cfg = ks_inputs.CONFIGS[3]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"])
    ell, B, n_rot, seed = cfg["L"], cfg["batch"], cfg["n_rot"], cfg["seed"]
    ct = st.uniform(seed, 1, (B, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (cfg["dnum"], 2), list(range(ell + cfg["K"]))) for r in range(n_rot)]
    pts = [st.uniform(seed, 100 + r, (), list(range(ell + cfg["K"]))) for r in range(n_rot)]
    galois = ks_inputs.galois_elements(cfg["logN"], n_rot)
    out = torch.empty((B, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_mac_hoisted(st.ctx, ct, ell, galois, keys, pts, out, workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, B, n_rot))
    torch.cuda.synchronize()
    hk, hp = [host(k) for k in keys], [host(w) for w in pts]
    for b in (0, 17, 63):      # first chunk, chunk boundary + 1, last
        want = st.ref.rotate_mac_hoisted(host(ct[b])[None], galois, hk, hp, ell)
        assert_equal(out[b], want[0])
    assert _in_range(out[40].reshape(-1, ell, st.N), st.q)


def test_cfg3_bsgs_full_size():
    """Configuration 3's parameters through the two-level transform: 64 ciphertexts, 16 baby steps x 4 giant steps."""
    cfg = ks_inputs.CONFIGS[3]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"])
    ell, B, seed, n1, n2 = cfg["L"], cfg["batch"], cfg["seed"], 16, 4
    all_ids = list(range(ell + cfg["K"]))
    gal = ks_inputs.galois_elements(cfg["logN"], n1 + n2)
    baby, giant = [1] + gal[:n1 - 1], [1] + gal[n1:n1 + n2 - 1]
    key = lambda tid, g: None if g == 1 else st.uniform(seed, tid, (cfg["dnum"], 2), all_ids)
    bkeys = [key(10 + i, g) for i, g in enumerate(baby)]
    gkeys = [key(40 + i, g) for i, g in enumerate(giant)]
    pts = [[st.uniform(seed, 100 + g * n1 + b, (), all_ids) for b in range(n1)] for g in range(n2)]
    ct = st.uniform(seed, 1, (B, 2), list(range(ell)))
    out = torch.empty((B, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_bsgs_linear_transform(st.ctx, ct, ell, baby, bkeys, giant, gkeys, pts, out, workspace(st.ctx, K.KS_OP_BSGS, ell, B))
    torch.cuda.synchronize()
    h = lambda x: None if x is None else host(x)
    hb, hg, hp = [h(k) for k in bkeys], [h(k) for k in gkeys], [[h(w) for w in row] for row in pts]
    for b in (0, 33):
        want = st.ref.bsgs_linear_transform(host(ct[b])[None], baby, hb, giant, hg, hp, ell)
        assert_equal(out[b], want[0])
    assert _in_range(out[63].reshape(-1, ell, st.N), st.q)


# ---- the same workloads with the paper's word size (28-bit primes, residues in 32-bit words), as `bench.py --word-size 32`
# runs them.  Sampled items are recomputed by the reference; every other output is compared with what the 64-bit entry
# point of the library gives on the same residues (itself checked against the reference above and in the other files).

def _narrow(t):
    return None if t is None else t.to(torch.int32)


def _widen(t):
    return t.to(torch.int64) & 0xFFFFFFFF


def test_cfg4_batched_ntt_full_size_32bit_words():
    cfg = dict(ks_inputs.CONFIGS[4], bits=28)
    st = Setup(cfg["logN"], cfg["L"], 0, 1, bits=28)
    ids = list(range(cfg["L"]))
    x = st.uniform(cfg["seed"], 1, (cfg["batch"],), ids)
    y = _narrow(x)
    K.ntt_fwd_u32(st.ctx, y, ids)
    for b in (0, cfg["batch"] - 1):              # every modulus, two whole polynomials
        assert_equal(_widen(y[b]), st.ref.ntt_fwd(host(x[b])[None], ids)[0])
    y64 = x.clone()
    K.ntt_fwd(st.ctx, y64, ids)
    assert torch.equal(_widen(y), y64)
    K.ntt_inv_u32(st.ctx, y, ids)
    assert torch.equal(_widen(y), x)


def test_cfg3_rotations_full_size_32bit_words():
    cfg = ks_inputs.CONFIGS[3]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"], bits=28)
    ell, B, n_rot, seed = cfg["L"], cfg["batch"], cfg["n_rot"], cfg["seed"]
    ct = st.uniform(seed, 1, (B, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (cfg["dnum"], 2), list(range(ell + cfg["K"]))) for r in range(n_rot)]
    pts = [st.uniform(seed, 100 + r, (), list(range(ell + cfg["K"]))) for r in range(n_rot)]
    galois = ks_inputs.galois_elements(cfg["logN"], n_rot)
    ct32, keys32, pts32 = _narrow(ct), [_narrow(k) for k in keys], [_narrow(w) for w in pts]
    # one workspace for the 32-bit and the 64-bit entry points: the larger of the two
    op = max((K.KS_OP_ROTATE_HOISTED_U32, K.KS_OP_ROTATE_HOISTED), key=lambda o: K.ks_workspace_bytes(st.ctx, o, ell, B, n_rot))
    ws = workspace(st.ctx, op, ell, B, n_rot)
    # hoisted rotations: 12 GiB of results in 32-bit words
    out32 = torch.empty((B, n_rot, 2, ell, st.N), dtype=torch.int32, device="cuda")
    K.ks_rotate_hoisted_u32(st.ctx, ct32, ell, galois, keys32, out32, ws)
    for b, r in [(0, 0), (17, 5), (63, 15)]:
        want = st.ref.rotate_hoisted(host(ct[b])[None], [galois[r]], [host(keys[r])], ell)
        assert_equal(_widen(out32[b, r]), want[0, 0])
    out64 = torch.empty((8, n_rot, 2, ell, st.N), dtype=torch.int64, device="cuda")
    for b0 in range(0, B, 8):                     # the 64-bit entry point on the same residues, a chunk at a time
        K.ks_rotate_hoisted(st.ctx, ct[b0:b0 + 8], ell, galois, keys, out64, ws)
        assert torch.equal(_widen(out32[b0:b0 + 8]), out64), b0
    del out32, out64
    # rotate-multiply-accumulate
    mac32 = torch.empty((B, 2, ell, st.N), dtype=torch.int32, device="cuda")
    K.ks_rotate_mac_hoisted_u32(st.ctx, ct32, ell, galois, keys32, pts32, mac32, ws)
    hk, hp = [host(k) for k in keys], [host(w) for w in pts]
    for b in (0, 63):
        assert_equal(_widen(mac32[b]), st.ref.rotate_mac_hoisted(host(ct[b])[None], galois, hk, hp, ell)[0])
    mac64 = torch.empty((B, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_mac_hoisted(st.ctx, ct, ell, galois, keys, pts, mac64, ws)
    assert torch.equal(_widen(mac32), mac64)


@pytest.mark.parametrize("merged", [False, True])
def test_cfg5_hmult_full_size_32bit_words(merged):
    cfg = ks_inputs.CONFIGS[5]
    st = Setup(cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"], bits=28)
    ell, B, seed = cfg["L"], cfg["batch"], cfg["seed"]
    cta = st.uniform(seed, 1, (B, 2), list(range(ell)))
    ctb = st.uniform(seed, 2, (B, 2), list(range(ell)))
    rlk = st.uniform(seed, 3, (cfg["dnum"], 2), list(range(ell + cfg["K"])))
    ws = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, B)
    out32 = torch.empty((B, 2, ell - 1, st.N), dtype=torch.int32, device="cuda")
    out64 = torch.empty((B, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
    if merged:
        K.hmult_relin_rescale_merged_u32(st.ctx, _narrow(cta), _narrow(ctb), ell, _narrow(rlk), out32, ws)
        K.hmult_relin_rescale_merged(st.ctx, cta, ctb, ell, rlk, out64, ws)
        ref = st.ref.hmult_relin_rescale_merged
    else:
        K.hmult_relin_rescale_u32(st.ctx, _narrow(cta), _narrow(ctb), ell, _narrow(rlk), out32, ws)
        K.hmult_relin_rescale(st.ctx, cta, ctb, ell, rlk, out64, ws)
        ref = st.ref.hmult_relin_rescale
    for b in (0, 16, 255):
        assert_equal(_widen(out32[b]), ref(host(cta[b])[None], host(ctb[b])[None], host(rlk), ell)[0])
    assert torch.equal(_widen(out32), out64)
