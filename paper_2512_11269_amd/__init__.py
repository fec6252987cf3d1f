"""MI355X-native CKKS hybrid key-switching: thin Python binding over the C-ABI library."""

from .binding import (  # noqa: F401
    KS_OP_BSGS,
    KS_OP_HMULT_RELIN_RESCALE,
    KS_OP_KEYSWITCH,
    KS_OP_ROTATE_HOISTED,
    Context,
    KsError,
    bconv,
    hmult_relin_rescale,
    hmult_relin_rescale_merged,
    ks_bsgs_linear_transform,
    ks_keyswitch,
    ks_profile_enable,
    ks_profile_report,
    ks_rotate_hoisted,
    ks_rotate_mac_hoisted,
    ks_workspace_bytes,
    library_path,
    load_library,
    ntt_fwd,
    ntt_inv,
)
