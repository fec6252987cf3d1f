"""ks_keyswitch_static (workspace = the library's static device array, nothing allocated) against ks_keyswitch
(workspace passed by the caller): identical residues, on calls in a row that share the array -- the later ones
smaller than the first, so stale contents of the array lie beside and behind what they use."""

import pytest
import torch

import paper_2512_11269_amd as K
from gpu_util import Setup, workspace

pytestmark = pytest.mark.gpu


def _both(st, seed, ell, batch):
    d = st.uniform(seed, 1, (batch,), list(range(ell)))
    evk = st.uniform(seed, 2, (st.ctx.dnum, 2), list(range(st.L + st.K)))
    want = torch.empty((batch, 2, ell, st.N), dtype=torch.int64, device="cuda")
    K.ks_keyswitch(st.ctx, d, ell, evk, want, workspace(st.ctx, K.KS_OP_KEYSWITCH, ell, batch))
    got = torch.full_like(want, -1)
    K.ks_keyswitch_static(st.ctx, d, ell, evk, got)
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_keyswitch_matches_workspace_keyswitch():
    boot = Setup(16, 24, 8, 3)       # configuration 2: one ciphertext fills the static array exactly
    assert K.ks_workspace_bytes(boot.ctx, K.KS_OP_KEYSWITCH, 24, 1) == K.ks_static_workspace_bytes()
    got, want = _both(boot, 41, 24, 1)
    assert torch.equal(got, want)
    small = Setup(12, 4, 2, 2)       # configuration 1's parameters on the same array, right after
    got, want = _both(small, 42, 4, 3)
    assert torch.equal(got, want)
    got, want = _both(small, 43, 3, 1)   # smaller again: lower level, one ciphertext
    assert torch.equal(got, want)
    got, want = _both(boot, 44, 17, 1)   # and back to the large ring at a lower level (short last digit)
    assert torch.equal(got, want)


def test_static_scratch_rejects_oversize():
    boot = Setup(16, 24, 8, 3)
    d = boot.uniform(45, 1, (2,), list(range(24)))
    evk = boot.uniform(45, 2, (3, 2), list(range(32)))
    out = torch.empty((2, 2, 24, boot.N), dtype=torch.int64, device="cuda")
    with pytest.raises(K.KsError, match="workspace"):
        K.ks_keyswitch_static(boot.ctx, d, 24, evk, out)   # two ciphertexts need twice the array
