"""The two base-conversion kernel families -- vector fp64 accumulation and int8 matrix cores (one or three targets per
lane half) -- forced through the context option, each against the plain-C reference, bit-exact on every residue: the
standalone conversion, and the fused conversion + column transform inside ks_keyswitch / hmult_relin_rescale_merged.
Source counts 1 .. 13 cover every operand-slot shape of the matrix-core tables (1, 2 or 3 instructions per position, 1..3
sources per slot), including digits of different sizes in one launch."""

import pytest
import torch

import paper_2512_11269_amd as K
from gpu_util import Setup, assert_equal, host, workspace

pytestmark = pytest.mark.gpu

KERNELS = [(1, 0), (2, 1), (2, 3)]     # (KS_OPT_BCONV_KERNEL, KS_OPT_BCONV_TARGETS)


def _select(st, kernel, targets):
    st.ctx.set_option(K.KS_OPT_BCONV_KERNEL, kernel)
    st.ctx.set_option(K.KS_OPT_BCONV_TARGETS, targets)


@pytest.fixture(scope="module")
def small():
    return Setup(12, 9, 3, 3)        # digits of 3 limbs; 12 moduli to draw conversions from


@pytest.fixture(scope="module")
def boot():
    return Setup(16, 24, 8, 3)


@pytest.mark.parametrize("kernel,targets", KERNELS)
@pytest.mark.parametrize("which,src,dst,batch", [
    ("small", [4], [0, 11], 2),
    ("small", [0, 1], [2, 3, 4, 5, 6, 7, 8], 1),
    ("small", [9, 10, 11], list(range(9)), 3),
    ("small", [0, 2, 4, 6, 8], [1, 3, 5, 7, 9, 10, 11], 1),
    ("small", list(range(7)), [7, 8, 9, 10, 11], 2),
    ("small", list(range(1, 11)), [0, 11], 1),
    ("boot", list(range(8)), list(range(8, 32)), 2),
    ("boot", list(range(24, 32)), list(range(24)), 1),
    ("boot", list(range(13)), list(range(13, 32)), 1),
    ("boot", list(range(16, 32)), [0, 5, 15], 1),
])
def test_standalone_conversion(kernel, targets, which, src, dst, batch, request):
    st = request.getfixturevalue(which)
    _select(st, kernel, targets)
    x = st.uniform(31, 2, (batch,), src)
    out = torch.full((batch, len(dst), st.N), -1, dtype=torch.int64, device="cuda")
    K.bconv_prepare(st.ctx, src, dst)
    K.bconv(st.ctx, x, src, out, dst)
    assert_equal(out, st.ref.bconv(host(x), src, dst))


def test_standalone_conversion_extreme_residues(boot):
    """All-zero and all (modulus - 1) sources: the ends of the byte-cutting range."""
    src, dst = list(range(8)), list(range(8, 32))
    x = torch.zeros((2, 8, boot.N), dtype=torch.int64, device="cuda")
    for i, m in enumerate(src):
        x[1, i, :] = boot.moduli[m] - 1
    K.bconv_prepare(boot.ctx, src, dst)
    for kernel, targets in KERNELS:
        _select(boot, kernel, targets)
        out = torch.full((2, 24, boot.N), -1, dtype=torch.int64, device="cuda")
        K.bconv(boot.ctx, x, src, out, dst)
        assert_equal(out, boot.ref.bconv(host(x), src, dst))
        assert int(out[0].abs().max()) == 0


@pytest.mark.parametrize("kernel,targets", KERNELS)
@pytest.mark.parametrize("logN,L,Kk,dnum,ells", [
    (12, 5, 2, 3, (5, 4, 1)),        # digits 2 / 2 / 1
    (12, 9, 3, 3, (9, 7)),           # 3-limb digits, short last digit at level 7
    (12, 6, 6, 1, (6, 5)),           # one digit of 6 (and 7 sources in the merged ModDown)
    (13, 4, 2, 2, (4,)),
    (14, 6, 3, 2, (6,)),
    (15, 4, 2, 2, (3,)),
    (16, 24, 8, 3, (24, 17)),        # configuration 2; level 17 has digits 8 / 8 / 1
    (16, 13, 13, 1, (13,)),          # 13 sources: three matrix instructions per position
])
def test_fused_conversion_in_keyswitch(kernel, targets, logN, L, Kk, dnum, ells):
    st = Setup(logN, L, Kk, dnum)
    _select(st, kernel, targets)
    evk = st.uniform(32, 2, (dnum, 2), list(range(L + Kk)))
    for ell in ells:
        batch = 1 if logN == 16 else 3
        d = st.uniform(32, 10 + ell, (batch,), list(range(ell)))
        out = torch.full((batch, 2, ell, st.N), -1, dtype=torch.int64, device="cuda")
        K.ks_keyswitch(st.ctx, d, ell, evk, out, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch))
        assert_equal(out, st.ref.keyswitch(host(d), host(evk), ell))


@pytest.mark.parametrize("kernel,targets", KERNELS)
def test_fused_conversion_in_merged_multiplication(kernel, targets):
    st = Setup(12, 6, 6, 1)
    _select(st, kernel, targets)
    rlk = st.uniform(33, 3, (1, 2), list(range(12)))
    for ell in (6, 3):
        cta = st.uniform(33, 20 + ell, (2, 2), list(range(ell)))
        ctb = st.uniform(33, 40 + ell, (2, 2), list(range(ell)))
        out = torch.full((2, 2, ell - 1, st.N), -1, dtype=torch.int64, device="cuda")
        K.hmult_relin_rescale_merged(st.ctx, cta, ctb, ell, rlk, out, workspace(st.ctx, K.KS_OP_HMULT_RELIN_RESCALE, ell, 2))
        assert_equal(out, st.ref.hmult_relin_rescale_merged(host(cta), host(ctb), host(rlk), ell))


def test_option_values_are_checked(small):
    with pytest.raises(K.KsError):
        small.ctx.set_option(K.KS_OPT_BCONV_KERNEL, 3)
    with pytest.raises(K.KsError):
        small.ctx.set_option(99, 0)
    small.ctx.set_option(K.KS_OPT_BCONV_KERNEL, 0)
    small.ctx.set_option(K.KS_OPT_BCONV_TARGETS, 0)
