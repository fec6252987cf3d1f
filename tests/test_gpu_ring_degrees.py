"""GPU parity at the ring degrees between the two benchmarked ones (N = 2^13, 2^14, 2^15: 32, 64 and 128 rows per limb, whose
column passes end with a shortened second register pass): transforms, base conversion and every pipeline entry point
against the plain-C reference, bit-exact on every residue."""

import pytest
import torch

import ks_inputs
import paper_2512_11269_amd as K
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=[13, 14, 15], ids=lambda n: "N2^%d" % n)
def st(request):
    return Setup(request.param, 5, 2, 3)     # digits 2 / 2 / 1


def test_transforms_and_conversion(st):
    ids = [0, 6, 3, 5]
    x = st.uniform(3001, 1, (3,), ids)
    y = x.clone()
    K.ntt_fwd(st.ctx, y, ids)
    assert_equal(y, st.ref.ntt_fwd(host(x), ids))
    K.ntt_inv(st.ctx, y, ids)
    assert torch.equal(y, x)
    w = x.clone()
    K.ntt_inv(st.ctx, w, ids)
    assert_equal(w, st.ref.ntt_inv(host(x), ids))
    src, dst = [5, 6], [0, 1, 2, 3, 4]
    xin = st.uniform(3001, 2, (2,), src)
    out = torch.empty((2, len(dst), st.N), dtype=torch.int64, device="cuda")
    K.bconv_prepare(st.ctx, src, dst)
    K.bconv(st.ctx, xin, src, out, dst)
    assert_equal(out, st.ref.bconv(host(xin), src, dst))


def test_pipelines(st):
    all_ids = list(range(st.L + st.K))
    evk = st.uniform(3002, 2, (st.ctx.dnum, 2), all_ids)
    gal = ks_inputs.galois_elements(st.logN, 3)
    keys = [st.uniform(3002, 50 + r, (st.ctx.dnum, 2), all_ids) for r in range(3)]
    pts = [st.uniform(3002, 70 + r, (), all_ids) for r in range(3)]
    for ell, batch in ((5, 9), (3, 2)):
        d = st.uniform(3002, 10 + ell, (batch,), list(range(ell)))
        out = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
        K.ks_keyswitch(st.ctx, d, ell, evk, out, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch))
        assert_equal(out, st.ref.keyswitch(host(d), host(evk), ell))
        ct = st.uniform(3002, 20 + ell, (batch, 2), list(range(ell)))
        ctb = st.uniform(3002, 30 + ell, (batch, 2), list(range(ell)))
        hw = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, batch)
        hout = torch.empty((batch, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
        K.hmult_relin_rescale(st.ctx, ct, ctb, ell, evk, hout, hw)
        assert_equal(hout, st.ref.hmult_relin_rescale(host(ct), host(ctb), host(evk), ell))
        K.hmult_relin_rescale_merged(st.ctx, ct, ctb, ell, evk, hout, hw)
        assert_equal(hout, st.ref.hmult_relin_rescale_merged(host(ct), host(ctb), host(evk), ell))
        rw = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, 3)
        rout = torch.empty((batch, 3, 2, ell, st.N), dtype=torch.int64, device="cuda")
        K.ks_rotate_hoisted(st.ctx, ct, ell, gal, keys, rout, rw)
        assert_equal(rout, st.ref.rotate_hoisted(host(ct), gal, [host(k) for k in keys], ell))
        K.ks_rotate_mac_hoisted(st.ctx, ct, ell, gal, keys, pts, out, rw)
        assert_equal(out, st.ref.rotate_mac_hoisted(host(ct), gal, [host(k) for k in keys], [host(w) for w in pts], ell))
