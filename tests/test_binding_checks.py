"""The Python binding refuses tensors whose sizes do not match what the header documents, before anything reaches the
library: the C ABI sees bare pointers, so an undersized output or key would become an out-of-bounds access on the GPU.
The checks depend only on element counts, so they are exercised here with CPU tensors and a stand-in context."""

import pytest
import torch

import paper_2512_11269_amd as K


class _Ctx:      # the attributes the wrappers read; no library handle, so nothing can be launched
    logN, N, L, K, dnum, device, handle = 12, 4096, 4, 2, 2, 0, None
    q, p = [0] * 4, [0] * 2


def _t(*shape, dtype=torch.int64):
    return torch.zeros(shape, dtype=dtype)


def _i(*shape):
    return _t(*shape, dtype=torch.int32)


CTX = _Ctx()
N = CTX.N
KEY = (2, 2, 6, N)


@pytest.mark.parametrize("call", [
    lambda: K.ks_keyswitch(CTX, _t(1, 4, N), 4, _t(*KEY), _t(1, 2, 3, N), _t(10)),                 # output one limb short
    lambda: K.ks_keyswitch(CTX, _t(1, 4, N - 1), 4, _t(*KEY), _t(1, 2, 4, N), _t(10)),             # d not a whole item
    lambda: K.ks_keyswitch(CTX, _t(1, 4, N), 4, _t(2, 2, 5, N), _t(1, 2, 4, N), _t(10)),           # key too small
    lambda: K.ks_keyswitch(CTX, _t(1, 5, N), 5, _t(*KEY), _t(1, 2, 5, N), _t(10)),                 # level above L
    lambda: K.ks_keyswitch(CTX, _t(0, 4, N), 4, _t(*KEY), _t(0, 2, 4, N), _t(10)),                 # empty batch
    lambda: K.ks_keyswitch_u32(CTX, _t(1, 4, N, dtype=torch.int32), 4, _t(*KEY, dtype=torch.int32), _t(1, 2, 2, N, dtype=torch.int32), _t(10)),
    lambda: K.ks_keyswitch_static(CTX, _t(1, 4, N), 4, _t(*KEY), _t(1, 1, 4, N)),
    lambda: K.ks_rotate_hoisted(CTX, _t(2, 2, 4, N), 4, [5, 25], [_t(*KEY), _t(*KEY)], _t(2, 1, 2, 4, N), _t(10)),     # out for one rotation only
    lambda: K.ks_rotate_hoisted(CTX, _t(2, 2, 4, N), 4, [5, 25], [_t(*KEY)], _t(2, 2, 2, 4, N), _t(10)),               # keys != elements
    lambda: K.ks_rotate_hoisted(CTX, _t(2, 2, 4, N), 4, [5], [_t(2, 2, 6, N // 2)], _t(2, 1, 2, 4, N), _t(10)),        # short key
    lambda: K.ks_rotate_mac_hoisted(CTX, _t(1, 2, 4, N), 4, [5], [_t(*KEY)], [_t(5, N)], _t(1, 2, 4, N), _t(10)),      # short plaintext
    lambda: K.ks_rotate_mac_hoisted(CTX, _t(1, 2, 4, N), 4, [5], [_t(*KEY)], [None, None], _t(1, 2, 4, N), _t(10)),
    lambda: K.ks_bsgs_linear_transform(CTX, _t(1, 2, 4, N), 4, [1, 5], [None, _t(*KEY)], [1], [None], [[None]], _t(1, 2, 4, N), _t(10)),
    lambda: K.hmult_relin_rescale(CTX, _t(1, 2, 4, N), _t(1, 2, 4, N), 4, _t(*KEY), _t(1, 2, 4, N), _t(10)),           # out must drop a limb
    lambda: K.hmult_relin_rescale(CTX, _t(2, 2, 4, N), _t(1, 2, 4, N), 4, _t(*KEY), _t(2, 2, 3, N), _t(10)),           # ctb smaller than cta
    lambda: K.hmult_relin_rescale_merged(CTX, _t(1, 2, 1, N), _t(1, 2, 1, N), 1, _t(*KEY), _t(1, 2, 0, N), _t(10)),    # level 1 cannot rescale
    lambda: K.ntt_fwd(CTX, _t(3, N - 8), [0, 1, 2]),
    lambda: K.ntt_inv(CTX, _t(2, N), [0, 1, 2]),
    lambda: K.bconv(CTX, _t(1, 2, N), [0, 1], _t(1, 3, N), [2, 3, 4, 5]),                          # output for three targets, four asked
    # the 32-bit-word forms check the same element counts
    lambda: K.ks_rotate_hoisted_u32(CTX, _i(2, 2, 4, N), 4, [5, 25], [_i(*KEY), _i(*KEY)], _i(2, 1, 2, 4, N), _t(10)),
    lambda: K.ks_rotate_mac_hoisted_u32(CTX, _i(1, 2, 4, N), 4, [5], [_i(*KEY)], [_i(5, N)], _i(1, 2, 4, N), _t(10)),
    lambda: K.ks_bsgs_linear_transform_u32(CTX, _i(1, 2, 4, N), 4, [1, 5], [None, _i(*KEY)], [1], [None], [[None]], _i(1, 2, 4, N), _t(10)),
    lambda: K.hmult_relin_rescale_u32(CTX, _i(1, 2, 4, N), _i(1, 2, 4, N), 4, _i(*KEY), _i(1, 2, 4, N), _t(10)),
    lambda: K.hmult_relin_rescale_merged_u32(CTX, _i(2, 2, 4, N), _i(1, 2, 4, N), 4, _i(*KEY), _i(2, 2, 3, N), _t(10)),
    lambda: K.ntt_fwd_u32(CTX, _i(3, N - 8), [0, 1, 2]),
    lambda: K.ntt_inv_u32(CTX, _i(2, N), [0, 1, 2]),
    lambda: K.bconv_u32(CTX, _i(1, 2, N), [0, 1], _i(1, 3, N), [2, 3, 4, 5]),
])
def test_wrong_sizes_are_refused(call):
    with pytest.raises(K.KsError):
        call()


def test_right_sizes_get_past_the_size_checks():
    """With consistent sizes the only remaining objection is that these are CPU tensors."""
    with pytest.raises(K.KsError, match="context on cuda"):
        K.ks_keyswitch(CTX, _t(3, 4, N), 4, _t(*KEY), _t(3, 2, 4, N), _t(10))
    with pytest.raises(K.KsError, match="context on cuda"):
        K.hmult_relin_rescale(CTX, _t(1, 2, 4, N), _t(1, 2, 4, N), 4, _t(*KEY), _t(1, 2, 3, N), _t(10))
