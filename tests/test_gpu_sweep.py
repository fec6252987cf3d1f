"""GPU parity sweep over parameter sets and every level at N = 2^12: digit partitions with short last digits, one digit,
one limb per digit, K different from alpha, every level ell from 1 (or 2) to L, batches across the chunk size.  Every entry
point of the pipeline family against the plain-C reference, bit-exact on every residue."""

import pytest
import torch

import ks_inputs
import paper_2512_11269_amd as K
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu

PARAMS = [(5, 2, 3), (6, 3, 2), (7, 1, 7), (3, 3, 1), (8, 4, 2), (9, 2, 4), (6, 6, 1)]   # (L, K, dnum)


@pytest.fixture(scope="module", params=PARAMS, ids=lambda p: "L%d-K%d-dnum%d" % p)
def st(request):
    L, Kk, dnum = request.param
    return Setup(12, L, Kk, dnum)


def _h(x):
    return None if x is None else host(x)


def test_keyswitch_every_level(st):
    all_ids = list(range(st.L + st.K))
    evk = st.uniform(2001, 2, (st.ctx.dnum, 2), all_ids)
    for ell in range(1, st.L + 1):
        batch = 1 + (ell * 5) % 11                       # 1 .. 11: below, at and above the chunk of 8
        d = st.uniform(2001, 10 + ell, (batch,), list(range(ell)))
        out = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
        K.ks_keyswitch(st.ctx, d, ell, evk, out, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch))
        assert_equal(out, st.ref.keyswitch(host(d), host(evk), ell))


def test_hmult_both_variants_every_level(st):
    all_ids = list(range(st.L + st.K))
    rlk = st.uniform(2002, 3, (st.ctx.dnum, 2), all_ids)
    for ell in range(2, st.L + 1):
        batch = 1 + ell % 3
        cta = st.uniform(2002, 20 + ell, (batch, 2), list(range(ell)))
        ctb = st.uniform(2002, 40 + ell, (batch, 2), list(range(ell)))
        ws = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, batch)
        out = torch.empty((batch, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
        K.hmult_relin_rescale(st.ctx, cta, ctb, ell, rlk, out, ws)
        assert_equal(out, st.ref.hmult_relin_rescale(host(cta), host(ctb), host(rlk), ell))
        K.hmult_relin_rescale_merged(st.ctx, cta, ctb, ell, rlk, out, ws)
        assert_equal(out, st.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), ell))


def test_rotations_every_level(st):
    all_ids = list(range(st.L + st.K))
    gal = ks_inputs.galois_elements(st.logN, 5)
    keys = [st.uniform(2003, 50 + r, (st.ctx.dnum, 2), all_ids) for r in range(5)]
    pts = [st.uniform(2003, 70 + r, (), all_ids) for r in range(5)]
    for ell in range(1, st.L + 1):
        batch = 1 + ell % 2
        ct = st.uniform(2003, 90 + ell, (batch, 2), list(range(ell)))
        ws = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, 5)
        out = torch.empty((batch, 5, 2, ell, st.N), dtype=torch.int64, device="cuda")
        K.ks_rotate_hoisted(st.ctx, ct, ell, gal, keys, out, ws)              # five rotations: a full group of four and one
        assert_equal(out, st.ref.rotate_hoisted(host(ct), gal, [host(k) for k in keys], ell))
        mac = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
        g2, k2, p2 = [1] + gal[:3], [None] + keys[:3], [pts[0], None, pts[2], pts[3]]
        K.ks_rotate_mac_hoisted(st.ctx, ct, ell, g2, k2, p2, mac, ws)
        assert_equal(mac, st.ref.rotate_mac_hoisted(host(ct), g2, [_h(k) for k in k2], [_h(w) for w in p2], ell))
        if ell in (1, st.L):
            K.ks_bsgs_linear_transform(st.ctx, ct, ell, g2[:2], k2[:2], [1, gal[4]], [None, keys[4]], [[pts[0], pts[1]], [None, pts[4]]],
                                       mac, workspace(st.ctx, K.KS_OP_BSGS, ell, batch))
            want = st.ref.bsgs_linear_transform(host(ct), g2[:2], [_h(k) for k in k2[:2]], [1, gal[4]], [None, host(keys[4])],
                                                [[host(pts[0]), host(pts[1])], [None, host(pts[4])]], ell)
            assert_equal(mac, want)
