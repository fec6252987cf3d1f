"""CPU-only checks of the boundary: the shared object loads, exports every function the header declares,
and rejects bad arguments before touching the GPU."""

import ctypes
import os
import re

import paper_2512_11269_amd as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ks.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = K.load_library()
    names = _declared_functions()
    assert {"ks_ctx_create", "ks_ctx_destroy", "ks_workspace_bytes", "ks_strerror", "ks_last_hip_error", "ntt_fwd",
            "ntt_inv", "bconv", "ks_keyswitch", "ks_rotate_hoisted", "hmult_relin_rescale", "hmult_relin_rescale_merged", "ks_rotate_mac_hoisted", "ks_bsgs_linear_transform", "ks_keyswitch_u32"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_ctx_create_rejects_bad_parameters_without_gpu():
    lib = K.load_library()
    h = ctypes.c_void_p()
    q_ok = (ctypes.c_uint64 * 2)(68719230977, 68719206401)      # = 1 mod 2^13, prime
    p_ok = (ctypes.c_uint64 * 1)(68719403009)
    bad_cases = [
        (11, 2, 1, 1, q_ok, p_ok),                               # unsupported ring degree
        (12, 0, 1, 1, q_ok, p_ok),                               # no ciphertext primes
        (12, 2, 1, 3, q_ok, p_ok),                               # dnum > L
        (12, 2, 1, 1, (ctypes.c_uint64 * 2)(68719230977, 68719230977), p_ok),   # repeated modulus
        (12, 2, 1, 1, (ctypes.c_uint64 * 2)(68719230977, 68719206401 + 8192), p_ok),  # composite (= 1 mod 2N)
        (12, 2, 1, 1, (ctypes.c_uint64 * 2)(68719230977, 97), p_ok),            # not 1 mod 2N
        (16, 2, 1, 1, q_ok, p_ok),                               # primes are 1 mod 2^13 but not mod 2^17
    ]
    for logN, L, Kk, dnum, q, p in bad_cases:
        assert lib.ks_ctx_create(ctypes.byref(h), logN, L, Kk, dnum, q, p, None, 0) == -1
        assert not h.value
    bad_psi = (ctypes.c_uint64 * 3)(2, 2, 2)
    assert lib.ks_ctx_create(ctypes.byref(h), 12, 2, 1, 1, q_ok, p_ok, bad_psi, 0) == -1
    assert lib.ks_strerror(-1).decode() == "invalid argument"
    assert lib.ks_strerror(-2).decode().startswith("workspace")


def test_null_context_is_rejected():
    lib = K.load_library()
    ids = (ctypes.c_uint32 * 1)(0)
    assert lib.ntt_fwd(None, None, ids, 1, 1, None) == -1
    assert lib.ks_keyswitch(None, None, 1, None, None, 1, None, 0, None) == -1
    assert lib.ks_workspace_bytes(None, 1, 1, 1, 0) == 0
