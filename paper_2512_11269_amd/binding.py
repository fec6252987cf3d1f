"""ctypes binding of libks_mi355x.so: argument marshalling only.

Functions carry the names of the C entry points (see include/ks.h) and take torch int64 CUDA tensors
laid out exactly as the header documents; torch provides device memory and the current HIP stream and
nothing else.  There is no fallback: if the shared object is missing or a call fails, an exception is
raised.
"""

from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# KS_MI355X_LIB selects another build of the same library (e.g. one compiled with different tuning macros)
_LIB_PATH = os.environ.get("KS_MI355X_LIB") or os.path.join(_HERE, "libks_mi355x.so")
_lib = None

KS_OP_KEYSWITCH, KS_OP_ROTATE_HOISTED, KS_OP_HMULT_RELIN_RESCALE, KS_OP_BSGS = 1, 2, 3, 4
KS_OPT_BCONV_TARGETS, KS_OPT_BCONV_KERNEL = 0, 1

_u64p = ctypes.POINTER(ctypes.c_uint64)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_vp = ctypes.c_void_p


class KsError(RuntimeError):
    pass


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built shared object (building it first only if none exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.ks_ctx_create.argtypes = [ctypes.POINTER(_vp), ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                  _u64p, _u64p, _u64p, ctypes.c_int]
    lib.ks_ctx_destroy.argtypes = [_vp]
    lib.ks_ctx_set_option.argtypes = [_vp, ctypes.c_int, ctypes.c_int]
    lib.ks_workspace_bytes.restype = ctypes.c_size_t
    lib.ks_workspace_bytes.argtypes = [_vp, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
    lib.ks_strerror.restype = ctypes.c_char_p
    lib.ks_strerror.argtypes = [ctypes.c_int]
    lib.ks_last_hip_error.restype = ctypes.c_char_p
    lib.ntt_fwd.argtypes = [_vp, _vp, _u32p, ctypes.c_uint32, ctypes.c_uint32, _vp]
    lib.ntt_inv.argtypes = [_vp, _vp, _u32p, ctypes.c_uint32, ctypes.c_uint32, _vp]
    lib.bconv_prepare.argtypes = [_vp, _u32p, ctypes.c_uint32, _u32p, ctypes.c_uint32]
    lib.bconv.argtypes = [_vp, _vp, _u32p, ctypes.c_uint32, _vp, _u32p, ctypes.c_uint32, ctypes.c_uint32, _vp]
    lib.ks_keyswitch.argtypes = [_vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.ks_keyswitch_u32.argtypes = [_vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.ks_static_workspace_bytes.restype = ctypes.c_size_t
    lib.ks_static_workspace_bytes.argtypes = []
    lib.ks_keyswitch_static.argtypes = [_vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint32, _vp]
    lib.ks_rotate_hoisted.argtypes = [_vp, _vp, ctypes.c_uint32, _u32p, ctypes.POINTER(_vp), ctypes.c_uint32, _vp,
                                      ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.ks_rotate_mac_hoisted.argtypes = [_vp, _vp, ctypes.c_uint32, _u32p, ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                          ctypes.c_uint32, _vp, ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.ks_bsgs_linear_transform.argtypes = [_vp, _vp, ctypes.c_uint32, _u32p, ctypes.POINTER(_vp), ctypes.c_uint32, _u32p,
                                             ctypes.POINTER(_vp), ctypes.c_uint32, ctypes.POINTER(_vp), _vp, ctypes.c_uint32, _vp,
                                             ctypes.c_size_t, _vp]
    lib.hmult_relin_rescale.argtypes = [_vp, _vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.hmult_relin_rescale_merged.argtypes = [_vp, _vp, _vp, ctypes.c_uint32, _vp, _vp, ctypes.c_uint32, _vp, ctypes.c_size_t, _vp]
    lib.ks_profile_enable.argtypes = [ctypes.c_int]
    lib.ks_profile_report.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    _lib = lib
    return lib


def ks_profile_enable(on: bool) -> None:
    _check(load_library().ks_profile_enable(1 if on else 0), "ks_profile_enable")


def ks_profile_report() -> list:
    """Per-kernel records [{kernel, launches, total_ms, total_bytes}] gathered since ks_profile_enable(True)."""
    import json
    buf = ctypes.create_string_buffer(1 << 16)
    _check(load_library().ks_profile_report(buf, len(buf)), "ks_profile_report")
    return json.loads(buf.value.decode())


def _check(rc: int, what: str):
    if rc != 0:
        lib = load_library()
        msg = lib.ks_strerror(rc).decode()
        if rc == -3:
            msg += ": " + lib.ks_last_hip_error().decode()
        raise KsError(f"{what} failed ({rc}): {msg}")


def _u64_array(values):
    return (ctypes.c_uint64 * len(values))(*[int(v) for v in values])


def _u32_array(values):
    return (ctypes.c_uint32 * len(values))(*[int(v) for v in values])


def _dev_ptr(t: torch.Tensor, dtype=torch.int64) -> int:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise KsError(f"expected a contiguous {dtype} CUDA tensor")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Context:
    """Owns a ks_ctx handle (device tables for one parameter set)."""

    def __init__(self, logN: int, q, p, dnum: int, psi=None, device: int = 0):
        lib = load_library()
        self.logN, self.N = logN, 1 << logN
        self.q, self.p = [int(x) for x in q], [int(x) for x in p]
        self.L, self.K, self.dnum = len(self.q), len(self.p), dnum
        self.device = device
        h = _vp()
        qa = _u64_array(self.q)
        pa = _u64_array(self.p) if self.K else None
        sa = _u64_array(psi) if psi is not None else None
        _check(lib.ks_ctx_create(ctypes.byref(h), logN, self.L, self.K, dnum, qa, pa, sa, device), "ks_ctx_create")
        self.handle = h

    def set_option(self, option: int, value: int) -> None:
        _check(load_library().ks_ctx_set_option(self.handle, option, value), "ks_ctx_set_option")

    def close(self):
        if getattr(self, "handle", None):
            load_library().ks_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ks_workspace_bytes(ctx: Context, op: int, ell: int, batch: int, n_rot: int = 0) -> int:
    return int(load_library().ks_workspace_bytes(ctx.handle, op, ell, batch, n_rot))


def ntt_fwd(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    """In place on data [batch][nlimbs][N]."""
    nl = len(mod_ids)
    batch = data.numel() // (nl * ctx.N)
    _check(load_library().ntt_fwd(ctx.handle, _dev_ptr(data), _u32_array(mod_ids), nl, batch, _stream()), "ntt_fwd")


def ntt_inv(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    nl = len(mod_ids)
    batch = data.numel() // (nl * ctx.N)
    _check(load_library().ntt_inv(ctx.handle, _dev_ptr(data), _u32_array(mod_ids), nl, batch, _stream()), "ntt_inv")


def bconv_prepare(ctx: Context, src_ids, dst_ids) -> None:
    """Set-up call: builds the constant table of this (source, target) list pair once; bconv needs it."""
    _check(load_library().bconv_prepare(ctx.handle, _u32_array(src_ids), len(src_ids), _u32_array(dst_ids), len(dst_ids)),
           "bconv_prepare")


def bconv(ctx: Context, x: torch.Tensor, src_ids, out: torch.Tensor, dst_ids) -> None:
    batch = x.numel() // (len(src_ids) * ctx.N)
    _check(load_library().bconv(ctx.handle, _dev_ptr(x), _u32_array(src_ids), len(src_ids), _dev_ptr(out),
                                _u32_array(dst_ids), len(dst_ids), batch, _stream()), "bconv")


def ks_keyswitch(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor, ws: torch.Tensor) -> None:
    batch = d.numel() // (ell * ctx.N)
    _check(load_library().ks_keyswitch(ctx.handle, _dev_ptr(d), ell, _dev_ptr(evk), _dev_ptr(out), batch, _dev_ptr(ws),
                                       ws.numel() * 8, _stream()), "ks_keyswitch")


def ks_static_workspace_bytes() -> int:
    return int(load_library().ks_static_workspace_bytes())


def ks_keyswitch_static(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor) -> None:
    """ks_keyswitch on the library's own static scratch array: no workspace argument, no allocation."""
    batch = d.numel() // (ell * ctx.N)
    _check(load_library().ks_keyswitch_static(ctx.handle, _dev_ptr(d), ell, _dev_ptr(evk), _dev_ptr(out), batch, _stream()),
           "ks_keyswitch_static")


def ks_rotate_hoisted(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, out: torch.Tensor, ws: torch.Tensor) -> None:
    batch = ct.numel() // (2 * ell * ctx.N)
    ptrs = (_vp * len(rot_keys))(*[_dev_ptr(k) for k in rot_keys])
    _check(load_library().ks_rotate_hoisted(ctx.handle, _dev_ptr(ct), ell, _u32_array(galois), ptrs, len(rot_keys),
                                            _dev_ptr(out), batch, _dev_ptr(ws), ws.numel() * 8, _stream()), "ks_rotate_hoisted")


def hmult_relin_rescale(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor, out: torch.Tensor,
                        ws: torch.Tensor) -> None:
    batch = cta.numel() // (2 * ell * ctx.N)
    _check(load_library().hmult_relin_rescale(ctx.handle, _dev_ptr(cta), _dev_ptr(ctb), ell, _dev_ptr(rlk), _dev_ptr(out),
                                              batch, _dev_ptr(ws), ws.numel() * 8, _stream()), "hmult_relin_rescale")


def hmult_relin_rescale_merged(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor, out: torch.Tensor,
                               ws: torch.Tensor) -> None:
    batch = cta.numel() // (2 * ell * ctx.N)
    _check(load_library().hmult_relin_rescale_merged(ctx.handle, _dev_ptr(cta), _dev_ptr(ctb), ell, _dev_ptr(rlk), _dev_ptr(out),
                                                     batch, _dev_ptr(ws), ws.numel() * 8, _stream()), "hmult_relin_rescale_merged")


def _ptr_array(tensors):
    """Host array of device pointers; None entries become NULL."""
    return (_vp * len(tensors))(*[None if t is None else _dev_ptr(t) for t in tensors])


def ks_rotate_mac_hoisted(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, pts, out: torch.Tensor, ws: torch.Tensor) -> None:
    batch = ct.numel() // (2 * ell * ctx.N)
    _check(load_library().ks_rotate_mac_hoisted(ctx.handle, _dev_ptr(ct), ell, _u32_array(galois), _ptr_array(rot_keys), _ptr_array(pts),
                                                len(rot_keys), _dev_ptr(out), batch, _dev_ptr(ws), ws.numel() * 8, _stream()),
           "ks_rotate_mac_hoisted")


def ks_bsgs_linear_transform(ctx: Context, ct: torch.Tensor, ell: int, baby_galois, baby_keys, giant_galois, giant_keys, pts,
                             out: torch.Tensor, ws: torch.Tensor) -> None:
    """pts: n2 rows of n1 plaintext tensors (or None)."""
    batch = ct.numel() // (2 * ell * ctx.N)
    flat = [w for row in pts for w in row]
    _check(load_library().ks_bsgs_linear_transform(ctx.handle, _dev_ptr(ct), ell, _u32_array(baby_galois), _ptr_array(baby_keys),
                                                   len(baby_keys), _u32_array(giant_galois), _ptr_array(giant_keys), len(giant_keys),
                                                   _ptr_array(flat), _dev_ptr(out), batch, _dev_ptr(ws), ws.numel() * 8, _stream()),
           "ks_bsgs_linear_transform")


def ks_keyswitch_u32(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor, ws: torch.Tensor) -> None:
    """d, evk, out: int32 tensors holding one residue (< 2^32) per 32-bit word; ws as for ks_keyswitch (int64)."""
    batch = d.numel() // (ell * ctx.N)
    _check(load_library().ks_keyswitch_u32(ctx.handle, _dev_ptr(d, torch.int32), ell, _dev_ptr(evk, torch.int32),
                                           _dev_ptr(out, torch.int32), batch, _dev_ptr(ws), ws.numel() * 8, _stream()), "ks_keyswitch_u32")
