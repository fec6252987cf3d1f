"""GPU parity: every entry point of the C-ABI library against the plain-C reference, bit-exact on every
residue, on seeded inputs spanning several tiles, ragged digits, lower levels and batch chunks."""

import numpy as np
import pytest
import torch

import ks_inputs
import paper_2512_11269_amd as K
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small():      # configuration 1: N = 2^12, L = 4, K = 2, dnum = 2
    return Setup(12, 4, 2, 2)


@pytest.fixture(scope="module")
def boot():       # configuration 2: N = 2^16, L = 24, K = 8, dnum = 3
    return Setup(16, 24, 8, 3)


@pytest.mark.parametrize("which,ids,batch", [("small", [0, 1, 2, 3, 4, 5, 0], 3), ("boot", [0, 31, 7, 24, 23], 2)])
def test_ntt_matches_reference_and_round_trips(which, ids, batch, request):
    st = request.getfixturevalue(which)
    x = st.uniform(7, 1, (batch,), ids)
    y = x.clone()
    K.ntt_fwd(st.ctx, y, ids)
    assert_equal(y, st.ref.ntt_fwd(host(x), ids))
    z = y.clone()
    K.ntt_inv(st.ctx, z, ids)
    assert torch.equal(z, x)
    w = x.clone()
    K.ntt_inv(st.ctx, w, ids)
    assert_equal(w, st.ref.ntt_inv(host(x), ids))


def test_ntt_edge_values(boot):
    """All-zero, all (m-1) and a single one: exercises the extremes of the lazy ranges."""
    ids = [0, 24, 31]
    N = boot.N
    x = torch.zeros((3, len(ids), N), dtype=torch.int64, device="cuda")
    for i, m in enumerate(ids):
        x[1, i, :] = boot.moduli[m] - 1
    x[2, :, 1] = 1
    y = x.clone()
    K.ntt_fwd(boot.ctx, y, ids)
    assert_equal(y, boot.ref.ntt_fwd(host(x), ids))
    assert int(y[0].abs().max()) == 0
    K.ntt_inv(boot.ctx, y, ids)
    assert torch.equal(y, x)


@pytest.mark.parametrize("which,src,dst,batch", [
    ("small", [0, 1], [2, 3, 4, 5], 2),
    ("small", [4, 5], [0, 1, 2, 3], 1),
    ("boot", list(range(8)), list(range(8, 32)), 2),
    ("boot", [16, 17, 18], [0, 1, 30, 31], 1),
    ("boot", [5], [0, 31], 1),
])
def test_bconv_matches_reference(which, src, dst, batch, request):
    st = request.getfixturevalue(which)
    x = st.uniform(8, 2, (batch,), src)
    out = torch.empty((batch, len(dst), st.N), dtype=torch.int64, device="cuda")
    K.bconv_prepare(st.ctx, src, dst)
    K.bconv(st.ctx, x, src, out, dst)
    assert_equal(out, st.ref.bconv(host(x), src, dst))
    out2 = torch.empty_like(out)
    K.bconv_prepare(st.ctx, src, dst)           # registering twice is harmless
    K.bconv(st.ctx, x, src, out2, dst)
    assert torch.equal(out, out2)


def test_bconv_needs_registration(small):
    """Compute calls never allocate: a conversion whose table was not built by bconv_prepare is refused."""
    x = small.uniform(8, 3, (1,), [1, 2])
    out = torch.empty((1, 1, small.N), dtype=torch.int64, device="cuda")
    with pytest.raises(K.KsError, match="not registered"):
        K.bconv(small.ctx, x, [1, 2], out, [5])


def _run_keyswitch(st, seed, ell, batch):
    d = st.uniform(seed, 1, (batch,), list(range(ell)))
    evk = st.uniform(seed, 2, (st.ctx.dnum, 2), list(range(st.L + st.K)))
    out = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch)
    K.ks_keyswitch(st.ctx, d, ell, evk, out, ws)
    return d, evk, out


@pytest.mark.parametrize("ell,batch", [(4, 1), (3, 2), (1, 1), (4, 19)])
def test_keyswitch_small(small, ell, batch):
    d, evk, out = _run_keyswitch(small, ks_inputs.CONFIGS[1]["seed"], ell, batch)
    assert_equal(out, small.ref.keyswitch(host(d), host(evk), ell))


@pytest.mark.parametrize("ell,batch", [(24, 1), (17, 2), (17, 1), (24, 9)])   # one ciphertext and several: different tile orders and load schedules; 9 = a chunk and one
def test_keyswitch_bootstrap_shape(boot, ell, batch):
    d, evk, out = _run_keyswitch(boot, ks_inputs.CONFIGS[2]["seed"], ell, batch)
    assert_equal(out, boot.ref.keyswitch(host(d), host(evk), ell))


def test_calls_are_deterministic(boot, small):
    """The same call twice into fresh outputs (and a fresh workspace) gives identical residues: no result depends on
    the order in which workgroups run or on what a buffer held before."""
    for st, ell in ((boot, 24), (small, 4)):
        d = st.uniform(91, 1, (2,), list(range(ell)))
        evk = st.uniform(91, 2, (st.ctx.dnum, 2), list(range(st.L + st.K)))
        outs = []
        for fill in (0, -1):
            out = torch.full((2, 2, ell, st.N), fill, dtype=torch.int64, device="cuda")
            ws = workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, 2)
            ws.fill_(fill)
            K.ks_keyswitch(st.ctx, d, ell, evk, out, ws)
            outs.append(out)
        assert torch.equal(outs[0], outs[1])
        cta, ctb = st.uniform(92, 3, (2, 2), list(range(ell))), st.uniform(92, 4, (2, 2), list(range(ell)))
        outs = []
        for fill in (0, -1):
            out = torch.full((2, 2, ell - 1, st.N), fill, dtype=torch.int64, device="cuda")
            ws = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, 2)
            ws.fill_(fill)
            K.hmult_relin_rescale(st.ctx, cta, ctb, ell, evk, out, ws)
            outs.append(out)
        assert torch.equal(outs[0], outs[1])


def test_keyswitch_zero_key_gives_zero(boot):
    d = boot.uniform(3, 1, (1,), list(range(24)))
    evk = torch.zeros((3, 2, 32, boot.N), dtype=torch.int64, device="cuda")
    out = torch.full((1, 2, 24, boot.N), -1, dtype=torch.int64, device="cuda")
    K.ks_keyswitch(boot.ctx, d, 24, evk, out, workspace(boot.ctx, K.KS_OP_KEYSWITCH, 24, 1))
    assert int(out.abs().max()) == 0


@pytest.mark.parametrize("logN,L,Kk,dnum,ell,batch", [(12, 4, 2, 2, 4, 3), (12, 5, 2, 3, 3, 9), (16, 24, 8, 3, 24, 2), (14, 6, 3, 2, 6, 1)])
def test_keyswitch_32bit_words(logN, L, Kk, dnum, ell, batch):
    """28-bit primes, boundary tensors in 32-bit words: same residues as the 64-bit entry point and as the reference."""
    st = Setup(logN, L, Kk, dnum, bits=28)
    assert max(st.moduli) < 1 << 28
    d = st.uniform(1010, 1, (batch,), list(range(ell)))
    evk = st.uniform(1010, 2, (dnum, 2), list(range(L + Kk)))
    ws = workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch)
    out32 = torch.empty((batch, 2, ell, st.N), dtype=torch.int32, device="cuda")
    K.ks_keyswitch_u32(st.ctx, d.to(torch.int32), ell, evk.to(torch.int32), out32, ws)
    want = st.ref.keyswitch(host(d), host(evk), ell)
    assert_equal(out32.to(torch.int64), want)
    out64 = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_keyswitch(st.ctx, d, ell, evk, out64, ws)
    assert torch.equal(out64, out32.to(torch.int64))


def test_keyswitch_32bit_words_needs_small_moduli(small):
    d = torch.zeros((1, 4, small.N), dtype=torch.int32, device="cuda")
    evk = torch.zeros((2, 2, 6, small.N), dtype=torch.int32, device="cuda")
    with pytest.raises(K.KsError):       # 36-bit moduli do not fit
        K.ks_keyswitch_u32(small.ctx, d, 4, evk, torch.empty((1, 2, 4, small.N), dtype=torch.int32, device="cuda"),
                           workspace(small.ctx, K.KS_OP_KEYSWITCH, 4, 1))


def test_keyswitch_is_capturable_in_a_graph(boot):
    """The entry points allocate nothing and never synchronise, so a call can be recorded into a HIP graph.  The graph is
    replayed several times with new inputs, eager calls and synchronisations in between; every replay must give what
    the eager call gives."""
    ell = 24
    d = boot.uniform(1011, 1, (2,), list(range(ell)))
    evk = boot.uniform(1011, 2, (3, 2), list(range(32)))
    out = torch.empty((2, 2, ell, boot.N), dtype=torch.int64, device="cuda")
    ws = workspace(boot.ctx, K.KS_OP_KEYSWITCH, ell, 2)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        K.ks_keyswitch(boot.ctx, d, ell, evk, out, ws)          # warm-up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            K.ks_keyswitch(boot.ctx, d, ell, evk, out, ws)
    torch.cuda.synchronize()
    eager_out, eager_ws = torch.empty_like(out), torch.empty_like(ws)
    for rep in range(3):
        d.copy_(boot.uniform(1011, 10 + rep, (2,), list(range(ell))))   # new input in the captured buffer
        K.ks_keyswitch(boot.ctx, d, ell, evk, eager_out, eager_ws)
        torch.cuda.synchronize()
        out.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out), rep
    assert_equal(out, boot.ref.keyswitch(host(d), host(evk), ell))


def _run_rotate(st, seed, ell, batch, n_rot):
    ct = st.uniform(seed, 1, (batch, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (st.ctx.dnum, 2), list(range(st.L + st.K))) for r in range(n_rot)]
    galois = ks_inputs.galois_elements(st.logN, n_rot)
    out = torch.empty((batch, n_rot, 2, ell, st.N), dtype=torch.int64, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n_rot)
    K.ks_rotate_hoisted(st.ctx, ct, ell, galois, keys, out, ws)
    return ct, keys, galois, out


@pytest.mark.parametrize("ell,batch,n_rot", [(4, 2, 3), (3, 1, 2)])
def test_rotate_hoisted_small(small, ell, batch, n_rot):
    ct, keys, galois, out = _run_rotate(small, 1003, ell, batch, n_rot)
    assert_equal(out, small.ref.rotate_hoisted(host(ct), galois, [host(k) for k in keys], ell))


def test_rotate_hoisted_bootstrap_shape(boot):
    ct, keys, galois, out = _run_rotate(boot, 1003, 24, 2, 2)
    assert_equal(out, boot.ref.rotate_hoisted(host(ct), galois, [host(k) for k in keys], 24))


def _run_rotate_mac(st, seed, ell, batch, n_rot):
    ct = st.uniform(seed, 1, (batch, 2), list(range(ell)))
    keys = [st.uniform(seed, 10 + r, (st.ctx.dnum, 2), list(range(st.L + st.K))) for r in range(n_rot)]
    pts = [st.uniform(seed, 100 + r, (), list(range(st.L + st.K))) for r in range(n_rot)]
    galois = ks_inputs.galois_elements(st.logN, n_rot)
    out = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n_rot)
    K.ks_rotate_mac_hoisted(st.ctx, ct, ell, galois, keys, pts, out, ws)
    return ct, keys, pts, galois, out


@pytest.mark.parametrize("ell,batch,n_rot", [(4, 2, 3), (3, 1, 2), (4, 19, 1), (4, 3, 18)])   # 18 rotations: two chained launches
def test_rotate_mac_small(small, ell, batch, n_rot):
    ct, keys, pts, galois, out = _run_rotate_mac(small, 1008, ell, batch, n_rot)
    assert_equal(out, small.ref.rotate_mac_hoisted(host(ct), galois, [host(k) for k in keys], [host(w) for w in pts], ell))


def test_rotate_mac_bootstrap_shape(boot):
    ct, keys, pts, galois, out = _run_rotate_mac(boot, 1008, 24, 2, 3)
    assert_equal(out, boot.ref.rotate_mac_hoisted(host(ct), galois, [host(k) for k in keys], [host(w) for w in pts], 24))


def test_rotate_mac_unit_plaintext_equals_rotate_hoisted(small):
    ell, g = 4, ks_inputs.galois_elements(small.logN, 2)[1]
    ct = small.uniform(6, 1, (2, 2), list(range(ell)))
    key = small.uniform(6, 2, (2, 2), list(range(6)))
    one = torch.ones((6, small.N), dtype=torch.int64, device="cuda")
    ws = workspace(small.ctx, K.KS_OP_ROTATE_HOISTED, ell, 2, 1)
    mac = torch.empty((2, 2, ell, small.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_mac_hoisted(small.ctx, ct, ell, [g], [key], [one], mac, ws)
    rot = torch.empty((2, 1, 2, ell, small.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_hoisted(small.ctx, ct, ell, [g], [key], rot, ws)
    assert torch.equal(mac, rot[:, 0])


def _bsgs_inputs(st, seed, ell, batch, n1, n2, with_identity=True):
    gal = ks_inputs.galois_elements(st.logN, n1 + n2)
    baby = ([1] if with_identity else []) + gal[:n1 - (1 if with_identity else 0)]
    giant = ([1] if with_identity else []) + gal[n1:n1 + n2 - (1 if with_identity else 0)]
    all_ids = list(range(st.L + st.K))
    key = lambda tid, g: None if g == 1 else st.uniform(seed, tid, (st.ctx.dnum, 2), all_ids)
    bkeys = [key(10 + i, g) for i, g in enumerate(baby)]
    gkeys = [key(40 + i, g) for i, g in enumerate(giant)]
    pts = [[st.uniform(seed, 100 + g * n1 + b, (), all_ids) for b in range(n1)] for g in range(n2)]
    pts[-1][0] = None                                        # a unit plaintext
    ct = st.uniform(seed, 1, (batch, 2), list(range(ell)))
    return ct, baby, bkeys, giant, gkeys, pts


def _hostify(x):
    return None if x is None else host(x)


@pytest.mark.parametrize("ell,batch,n1,n2", [(4, 2, 3, 2), (3, 17, 2, 3), (4, 1, 1, 1)])
def test_bsgs_small(small, ell, batch, n1, n2):
    ct, baby, bkeys, giant, gkeys, pts = _bsgs_inputs(small, 1009, ell, batch, n1, n2)
    out = torch.empty((batch, 2, ell, small.N), dtype=torch.int64, device="cuda")
    K.ks_bsgs_linear_transform(small.ctx, ct, ell, baby, bkeys, giant, gkeys, pts, out, workspace(small.ctx, K.KS_OP_BSGS, ell, batch))
    want = small.ref.bsgs_linear_transform(host(ct), baby, [_hostify(k) for k in bkeys], giant, [_hostify(k) for k in gkeys],
                                           [[_hostify(w) for w in row] for row in pts], ell)
    assert_equal(out, want)
    # the identity element and the unit plaintext through the single-level entry point
    mac = torch.empty_like(out)
    K.ks_rotate_mac_hoisted(small.ctx, ct, ell, baby, bkeys, pts[-1], mac, workspace(small.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n1))
    assert_equal(mac, small.ref.rotate_mac_hoisted(host(ct), baby, [_hostify(k) for k in bkeys], [_hostify(w) for w in pts[-1]], ell))


def test_bsgs_bootstrap_shape(boot):
    ct, baby, bkeys, giant, gkeys, pts = _bsgs_inputs(boot, 1009, 24, 2, 3, 2)
    out = torch.empty((2, 2, 24, boot.N), dtype=torch.int64, device="cuda")
    K.ks_bsgs_linear_transform(boot.ctx, ct, 24, baby, bkeys, giant, gkeys, pts, out, workspace(boot.ctx, K.KS_OP_BSGS, 24, 2))
    want = boot.ref.bsgs_linear_transform(host(ct), baby, [_hostify(k) for k in bkeys], giant, [_hostify(k) for k in gkeys],
                                          [[_hostify(w) for w in row] for row in pts], 24)
    assert_equal(out, want)


def test_rotate_by_identity_equals_keyswitch_plus_c0(small):
    ell = 4
    ct = small.uniform(5, 1, (1, 2), list(range(ell)))
    key = small.uniform(5, 2, (2, 2), list(range(6)))
    out = torch.empty((1, 1, 2, ell, small.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_hoisted(small.ctx, ct, ell, [1], [key], out, workspace(small.ctx, K.KS_OP_ROTATE_HOISTED, ell, 1, 1))
    ks = torch.empty((1, 2, ell, small.N), dtype=torch.int64, device="cuda")
    K.ks_keyswitch(small.ctx, ct[:, 1].contiguous(), ell, key, ks, workspace(small.ctx, K.KS_OP_KEYSWITCH, ell, 1))
    q = torch.tensor(small.q, dtype=torch.int64, device="cuda").view(ell, 1)
    assert torch.equal(out[0, 0, 1], ks[0, 1])
    assert torch.equal(out[0, 0, 0], (ks[0, 0] + ct[0, 0]) % q)


def _run_hmult(st, seed, ell, batch, merged=False):
    cta = st.uniform(seed, 1, (batch, 2), list(range(ell)))
    ctb = st.uniform(seed, 2, (batch, 2), list(range(ell)))
    rlk = st.uniform(seed, 3, (st.ctx.dnum, 2), list(range(st.L + st.K)))
    out = torch.empty((batch, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
    ws = workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, batch)
    (K.hmult_relin_rescale_merged if merged else K.hmult_relin_rescale)(st.ctx, cta, ctb, ell, rlk, out, ws)
    return cta, ctb, rlk, out


@pytest.mark.parametrize("ell,batch", [(4, 2), (2, 1), (4, 17)])
def test_hmult_small(small, ell, batch):
    cta, ctb, rlk, out = _run_hmult(small, 1005, ell, batch)
    assert_equal(out, small.ref.hmult_relin_rescale(host(cta), host(ctb), host(rlk), ell))


@pytest.mark.parametrize("ell,batch", [(4, 2), (2, 1), (3, 17)])
def test_hmult_merged_small(small, ell, batch):
    cta, ctb, rlk, out = _run_hmult(small, 1006, ell, batch, merged=True)
    assert_equal(out, small.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), ell))


def test_hmult_merged_llm_shape():
    st = Setup(16, 35, 12, 3)            # configuration 5 shape: 13 sources in the merged conversion
    cta, ctb, rlk, out = _run_hmult(st, 1006, 35, 2, merged=True)
    assert_equal(out, st.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), 35))
    cta, ctb, rlk, out = _run_hmult(st, 1007, 24, 1, merged=True)   # lower level: digits 12 / 12, short last source set
    assert_equal(out, st.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), 24))


def test_hmult_llm_shape():
    st = Setup(16, 35, 12, 3)            # configuration 5 shape: digits 12 / 12 / 11
    cta, ctb, rlk, out = _run_hmult(st, 1005, 35, 2)
    assert_equal(out, st.ref.hmult_relin_rescale(host(cta), host(ctb), host(rlk), 35))


def _boundary_residues(st, seed, lead, ids):
    """Residues drawn from the values around the cut of the packed 32 + 8 bit form (and the ends of the range):
    0, 1, 2^32 - 1, 2^32, 2^32 + 1, m - 2, m - 1 of each limb's modulus m."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    mods = torch.tensor([st.moduli[i] for i in ids], dtype=torch.int64)
    table = torch.stack([torch.zeros_like(mods), torch.ones_like(mods), torch.full_like(mods, 2**32 - 1), torch.full_like(mods, 2**32),
                         torch.full_like(mods, 2**32 + 1), mods - 2, mods - 1])          # [7][limbs]
    pick = torch.randint(0, 7, (*lead, len(ids), st.N), generator=g)
    limb = torch.arange(len(ids)).view(*([1] * len(lead)), len(ids), 1).expand_as(pick)
    return table[pick, limb].contiguous().cuda()


def test_pipelines_with_residues_at_the_packed_word_boundaries(small):
    """Intermediate tensors cross memory as a 32-bit word plus a byte per residue: inputs made of the values on both sides
    of that cut, through every pipeline that uses the packed form."""
    st, ell, batch = small, 4, 3
    assert min(st.moduli) > 2**32 + 1
    all_ids, ct_ids = list(range(st.L + st.K)), list(range(ell))
    d = _boundary_residues(st, 1, (batch,), ct_ids)
    evk = _boundary_residues(st, 2, (st.ctx.dnum, 2), all_ids)
    out = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_keyswitch(st.ctx, d, ell, evk, out, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch))
    assert_equal(out, st.ref.keyswitch(host(d), host(evk), ell))

    cta, ctb = _boundary_residues(st, 3, (batch, 2), ct_ids), _boundary_residues(st, 4, (batch, 2), ct_ids)
    for merged in (False, True):
        got = torch.empty((batch, 2, ell - 1, st.N), dtype=torch.int64, device="cuda")
        (K.hmult_relin_rescale_merged if merged else K.hmult_relin_rescale)(st.ctx, cta, ctb, ell, evk, got,
                                                                            workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, batch))
        ref = st.ref.hmult_relin_rescale_merged if merged else st.ref.hmult_relin_rescale
        assert_equal(got, ref(host(cta), host(ctb), host(evk), ell))

    n_rot = 3
    galois = ks_inputs.galois_elements(st.logN, n_rot)
    keys = [_boundary_residues(st, 10 + r, (st.ctx.dnum, 2), all_ids) for r in range(n_rot)]
    pts = [_boundary_residues(st, 20 + r, (), all_ids) for r in range(n_rot)]
    rot = torch.empty((batch, n_rot, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_hoisted(st.ctx, cta, ell, galois, keys, rot, workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n_rot))
    assert_equal(rot, st.ref.rotate_hoisted(host(cta), galois, [host(k) for k in keys], ell))
    mac = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_rotate_mac_hoisted(st.ctx, cta, ell, galois, keys, pts, mac, workspace(st.ctx, K.KS_OP_ROTATE_HOISTED, ell, batch, n_rot))
    assert_equal(mac, st.ref.rotate_mac_hoisted(host(cta), galois, [host(k) for k in keys], [host(w) for w in pts], ell))


def test_error_paths_return_codes(small):
    lib = K.load_library()
    ell = 4
    d = small.uniform(1, 1, (1,), list(range(ell)))
    evk = small.uniform(1, 2, (2, 2), list(range(6)))
    out = torch.empty((1, 2, ell, small.N), dtype=torch.int64, device="cuda")
    ws = workspace(small.ctx, K.KS_OP_KEYSWITCH, ell, 1)
    h = small.ctx.handle
    assert lib.ks_keyswitch(h, d.data_ptr(), 5, evk.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), ws.numel() * 8, None) == -1
    assert lib.ks_keyswitch(h, d.data_ptr(), ell, evk.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), 16, None) == -2
    assert lib.ks_keyswitch(h, d.data_ptr() + 8, ell, evk.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), ws.numel() * 8, None) == -1
    assert lib.ks_keyswitch(h, d.data_ptr(), ell, evk.data_ptr(), out.data_ptr(), 1, None, 0, None) == -2
    with pytest.raises(K.KsError):
        K.ks_rotate_hoisted(small.ctx, torch.zeros((1, 2, ell, small.N), dtype=torch.int64, device="cuda"), ell, [4], [evk],
                            torch.empty((1, 1, 2, ell, small.N), dtype=torch.int64, device="cuda"), ws)
    with pytest.raises(K.KsError):
        K.ntt_fwd(small.ctx, d, [99])
    ct = torch.zeros((1, 2, ell, small.N), dtype=torch.int64, device="cuda")
    pt = torch.ones((6, small.N), dtype=torch.int64, device="cuda")
    with pytest.raises(K.KsError):          # even Galois element
        K.ks_rotate_mac_hoisted(small.ctx, ct, ell, [6], [evk], [pt], out, ws)
    with pytest.raises(K.KsError):          # nothing to drop at one limb
        K.hmult_relin_rescale_merged(small.ctx, ct[:, :, :1].contiguous(), ct[:, :, :1].contiguous(), 1, evk,
                                     torch.empty((1, 2, 1, small.N), dtype=torch.int64, device="cuda"),
                                     workspace(small.ctx, K.KS_OP_HMULT_RELIN_RESCALE, 2, 1))
    # an empty batch is a no-op that succeeds and leaves the output alone
    out.fill_(-7)
    assert lib.ks_keyswitch(h, d.data_ptr(), ell, evk.data_ptr(), out.data_ptr(), 0, ws.data_ptr(), ws.numel() * 8, None) == 0
    assert lib.hmult_relin_rescale_merged(h, ct.data_ptr(), ct.data_ptr(), ell, evk.data_ptr(), out.data_ptr(), 0, ws.data_ptr(),
                                          ws.numel() * 8, None) == 0
    torch.cuda.synchronize()
    assert int((out != -7).sum()) == 0
    torch.cuda.synchronize()
