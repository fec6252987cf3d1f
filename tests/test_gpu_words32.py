"""The entry points that take their tensors in 32-bit words (Evaluation, "Benchmarks": a 28-bit RNS basis in 32-bit
words) against the C reference, residue for residue, and against the 64-bit entry points of the same library.

The reference has one word size (64 bits): the 32-bit tensors are the same residues narrowed on the device, results
are widened before the comparison.  28-bit moduli are the paper's; the 32-bit moduli exercise values with the top
bit of the word set."""

import pytest
import torch

import ks_inputs
import paper_2512_11269_amd as K
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu


def narrow(t):
    return None if t is None else t.to(torch.int32)


def widen(t):
    return t.to(torch.int64) & 0xFFFFFFFF


@pytest.fixture(scope="module")
def small28():
    return Setup(12, 4, 2, 2, bits=28)


@pytest.fixture(scope="module")
def small32():
    return Setup(12, 5, 2, 3, bits=32)


@pytest.fixture(scope="module")
def boot28():
    return Setup(16, 24, 8, 3, bits=28)   # configuration 2 shape with the paper's word size


@pytest.mark.parametrize("which,ids,batch", [("small28", [0, 1, 2, 3, 4, 5], 3), ("small32", [6, 0, 3], 2), ("boot28", [0, 7, 31], 2),
                                             ("boot28", list(range(32)), 1)])
def test_transforms(which, ids, batch, request):
    st = request.getfixturevalue(which)
    assert max(st.moduli) < 1 << (32 if which == "small32" else 28)
    x = st.uniform(2001, 1, (batch,), ids)
    y = narrow(x)
    K.ntt_fwd_u32(st.ctx, y, ids)
    assert_equal(widen(y), st.ref.ntt_fwd(host(x), ids))
    x64 = x.clone()
    K.ntt_fwd(st.ctx, x64, ids)
    assert torch.equal(widen(y), x64)
    K.ntt_inv_u32(st.ctx, y, ids)
    assert torch.equal(widen(y), x)
    z = narrow(x)
    K.ntt_inv_u32(st.ctx, z, ids)
    assert_equal(widen(z), st.ref.ntt_inv(host(x), ids))


@pytest.mark.parametrize("logN", [13, 14, 15])
def test_transforms_other_ring_degrees(logN):
    st = Setup(logN, 3, 1, 3, bits=28)
    ids = [0, 1, 2, 3]
    x = st.uniform(2002, 1, (2,), ids)
    y = narrow(x)
    K.ntt_fwd_u32(st.ctx, y, ids)
    assert_equal(widen(y), st.ref.ntt_fwd(host(x), ids))
    K.ntt_inv_u32(st.ctx, y, ids)
    assert torch.equal(widen(y), x)


def test_transform_edge_values(boot28):
    ids = [0, 31]
    mods = torch.tensor([boot28.moduli[i] for i in ids], dtype=torch.int64, device="cuda").view(1, 2, 1)
    x = (mods - 1).expand(1, 2, boot28.N).contiguous()           # every residue at its maximum
    y = narrow(x)
    K.ntt_fwd_u32(boot28.ctx, y, ids)
    assert_equal(widen(y), boot28.ref.ntt_fwd(host(x), ids))
    z = torch.zeros((1, 2, boot28.N), dtype=torch.int32, device="cuda")
    K.ntt_fwd_u32(boot28.ctx, z, ids)
    assert int(z.abs().max()) == 0


@pytest.mark.parametrize("which,src,dst,batch", [("small28", [0, 1], [2, 3, 4, 5], 3), ("small32", [5, 6], [0, 1, 2, 3, 4], 2),
                                                 ("boot28", list(range(8)), list(range(8, 32)), 2),
                                                 ("boot28", list(range(24, 32)), list(range(24)), 1)])
def test_conversion(which, src, dst, batch, request):
    st = request.getfixturevalue(which)
    x = st.uniform(2003, 1, (batch,), src)
    K.bconv_prepare(st.ctx, src, dst)
    out = torch.empty((batch, len(dst), st.N), dtype=torch.int32, device="cuda")
    K.bconv_u32(st.ctx, narrow(x), src, out, dst)
    assert_equal(widen(out), st.ref.bconv(host(x), src, dst))


def _rotation_inputs(st, seed, ell, batch, n_rot, with_pts):
    ct = st.uniform(seed, 1, (batch, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (st.ctx.dnum, 2), list(range(st.L + st.K))) for r in range(n_rot)]
    pts = [st.uniform(seed, 100 + r, (), list(range(st.L + st.K))) for r in range(n_rot)] if with_pts else None
    return ct, keys, pts, ks_inputs.galois_elements(st.logN, n_rot)


@pytest.mark.parametrize("which,ell,batch,n_rot", [("small28", 4, 2, 3), ("small32", 3, 9, 5), ("boot28", 24, 2, 2)])
def test_rotate_hoisted(which, ell, batch, n_rot, request):
    st = request.getfixturevalue(which)
    ct, keys, _, galois = _rotation_inputs(st, 2004, ell, batch, n_rot, False)
    out = torch.empty((batch, n_rot, 2, ell, st.N), dtype=torch.int32, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED_U32, ell, batch, n_rot)
    K.ks_rotate_hoisted_u32(st.ctx, narrow(ct), ell, galois, [narrow(k) for k in keys], out, ws)
    assert_equal(widen(out), st.ref.rotate_hoisted(host(ct), galois, [host(k) for k in keys], ell))


@pytest.mark.parametrize("which,ell,batch,n_rot", [("small28", 4, 2, 3), ("small32", 5, 3, 18), ("boot28", 24, 2, 3)])
def test_rotate_mac(which, ell, batch, n_rot, request):
    st = request.getfixturevalue(which)
    ct, keys, pts, galois = _rotation_inputs(st, 2005, ell, batch, n_rot, True)
    galois[0], keys[0] = 1, None        # the unrotated term: no key
    pts[-1] = None                      # a unit plaintext
    out = torch.empty((batch, 2, ell, st.N), dtype=torch.int32, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED_U32, ell, batch, n_rot)
    K.ks_rotate_mac_hoisted_u32(st.ctx, narrow(ct), ell, galois, [narrow(k) for k in keys], [narrow(w) for w in pts], out, ws)
    hostify = lambda t: None if t is None else host(t)
    assert_equal(widen(out), st.ref.rotate_mac_hoisted(host(ct), galois, [hostify(k) for k in keys], [hostify(w) for w in pts], ell))
    out64 = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_mac_hoisted(st.ctx, ct, ell, galois, keys, pts, out64, workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n_rot))
    assert torch.equal(out64, widen(out))


@pytest.mark.parametrize("merged", [False, True])
@pytest.mark.parametrize("which,ell,batch", [("small28", 4, 2), ("small28", 2, 1), ("small32", 5, 17), ("boot28", 24, 2)])
def test_multiplication(which, ell, batch, merged, request):
    st = request.getfixturevalue(which)
    cta = st.uniform(2006, 1, (batch, 2), list(range(ell)))
    ctb = st.uniform(2006, 2, (batch, 2), list(range(ell)))
    rlk = st.uniform(2006, 3, (st.ctx.dnum, 2), list(range(st.L + st.K)))
    out = torch.empty((batch, 2, ell - 1, st.N), dtype=torch.int32, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, batch)
    if merged:
        K.hmult_relin_rescale_merged_u32(st.ctx, narrow(cta), narrow(ctb), ell, narrow(rlk), out, ws)
        want = st.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), ell)
    else:
        K.hmult_relin_rescale_u32(st.ctx, narrow(cta), narrow(ctb), ell, narrow(rlk), out, ws)
        want = st.ref.hmult_relin_rescale(host(cta), host(ctb), host(rlk), ell)
    assert_equal(widen(out), want)


def test_wide_moduli_are_refused():
    st = Setup(12, 4, 2, 2)             # 36-bit moduli do not fit a 32-bit word
    N, i32 = st.N, dict(dtype=torch.int32, device="cuda")
    ct = torch.zeros((1, 2, 4, N), **i32)
    key = torch.zeros((2, 2, 6, N), **i32)
    with pytest.raises(K.KsError):
        K.ntt_fwd_u32(st.ctx, torch.zeros((1, 2, N), **i32), [0, 1])
    with pytest.raises(K.KsError):
        K.ntt_inv_u32(st.ctx, torch.zeros((1, 2, N), **i32), [0, 1])
    K.bconv_prepare(st.ctx, [0, 1], [2])
    with pytest.raises(K.KsError):
        K.bconv_u32(st.ctx, torch.zeros((1, 2, N), **i32), [0, 1], torch.zeros((1, 1, N), **i32), [2])
    with pytest.raises(K.KsError):
        K.ks_rotate_hoisted_u32(st.ctx, ct, 4, [5], [key], torch.zeros((1, 1, 2, 4, N), **i32),
                                workspace(st.ctx, K.KS_OP_ROTATE_HOISTED_U32, 4, 1, 1))
    with pytest.raises(K.KsError):
        K.ks_rotate_mac_hoisted_u32(st.ctx, ct, 4, [5], [key], [None], torch.zeros((1, 2, 4, N), **i32),
                                    workspace(st.ctx, K.KS_OP_ROTATE_HOISTED_U32, 4, 1, 1))
    for call in (K.hmult_relin_rescale_u32, K.hmult_relin_rescale_merged_u32):
        with pytest.raises(K.KsError):
            call(st.ctx, ct, ct, 4, key, torch.zeros((1, 2, 3, N), **i32), workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, 4, 1))


@pytest.mark.parametrize("targets,batch", [(0, 1), (1, 1), (2, 2), (3, 1), (4, 1), (0, 9)])
def test_two_piece_conversion_at_the_benchmarked_shape(boot28, targets, batch):
    """With every modulus below 2^32 the vector conversion kernel cuts a source residue into two pieces instead of
    three.  All of its launch shapes (targets per workgroup; 0 = the library's choice) at the configuration 2 shape."""
    ell = 24
    d = boot28.uniform(2007, 1, (batch,), list(range(ell)))
    evk = boot28.uniform(2007, 2, (3, 2), list(range(32)))
    out = torch.empty((batch, 2, ell, boot28.N), dtype=torch.int64, device="cuda")
    boot28.ctx.set_option(K.KS_OPT_BCONV_KERNEL, 1)
    boot28.ctx.set_option(K.KS_OPT_BCONV_TARGETS, targets)
    try:
        K.ks_keyswitch(boot28.ctx, d, ell, evk, out, workspace(boot28.ctx, K.KS_OP_KEYSWITCH, ell, batch))
    finally:
        boot28.ctx.set_option(K.KS_OPT_BCONV_KERNEL, 0)
        boot28.ctx.set_option(K.KS_OPT_BCONV_TARGETS, 0)
    assert_equal(out, boot28.ref.keyswitch(host(d), host(evk), ell))


@pytest.mark.parametrize("which", ["small28", "small32"])
def test_two_piece_conversion_extreme_residues(which, request):
    """Every source residue at modulus - 1 (the largest pieces) and at 0, through the vector conversion kernel; with
    32-bit moduli the exact sums come closest to the 2^53 they must stay below."""
    st = request.getfixturevalue(which)
    ell = st.L
    q = torch.tensor(st.q, dtype=torch.int64, device="cuda").view(1, ell, 1)
    evk = st.uniform(2008, 2, (st.ctx.dnum, 2), list(range(st.L + st.K)))
    for d in ((q - 1).expand(1, ell, st.N).contiguous(), torch.zeros((1, ell, st.N), dtype=torch.int64, device="cuda")):
        out = torch.empty((1, 2, ell, st.N), dtype=torch.int64, device="cuda")
        K.ks_keyswitch(st.ctx, d, ell, evk, out, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, 1))
        assert_equal(out, st.ref.keyswitch(host(d), host(evk), ell))


@pytest.mark.parametrize("which,ell,batch,n1,n2", [("small28", 4, 2, 3, 2), ("small32", 3, 9, 2, 3), ("boot28", 24, 2, 3, 2)])
def test_bsgs_linear_transform(which, ell, batch, n1, n2, request):
    """Both hoisting levels with keys, plaintexts, ciphertexts and result in 32-bit words; the identity element (no key)
    and a unit plaintext included."""
    st = request.getfixturevalue(which)
    gal = ks_inputs.galois_elements(st.logN, n1 + n2)
    baby, giant = [1] + gal[:n1 - 1], [1] + gal[n1:n1 + n2 - 1]
    all_ids = list(range(st.L + st.K))
    key = lambda tid, g: None if g == 1 else st.uniform(2009, tid, (st.ctx.dnum, 2), all_ids)
    bkeys = [key(10 + i, g) for i, g in enumerate(baby)]
    gkeys = [key(40 + i, g) for i, g in enumerate(giant)]
    pts = [[st.uniform(2009, 100 + g * n1 + b, (), all_ids) for b in range(n1)] for g in range(n2)]
    pts[-1][0] = None
    ct = st.uniform(2009, 1, (batch, 2), list(range(ell)))
    out = torch.empty((batch, 2, ell, st.N), dtype=torch.int32, device="cuda")
    K.ks_bsgs_linear_transform_u32(st.ctx, narrow(ct), ell, baby, [narrow(k) for k in bkeys], giant, [narrow(k) for k in gkeys],
                                   [[narrow(w) for w in row] for row in pts], out, workspace(st.ctx, K.KS_OP_BSGS_U32, ell, batch))
    hostify = lambda t: None if t is None else host(t)
    want = st.ref.bsgs_linear_transform(host(ct), baby, [hostify(k) for k in bkeys], giant, [hostify(k) for k in gkeys],
                                        [[hostify(w) for w in row] for row in pts], ell)
    assert_equal(widen(out), want)
