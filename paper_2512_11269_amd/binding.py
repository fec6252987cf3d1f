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

KS_OP_KEYSWITCH, KS_OP_ROTATE_HOISTED, KS_OP_HMULT_RELIN_RESCALE, KS_OP_BSGS, KS_OP_ROTATE_HOISTED_U32, KS_OP_BSGS_U32 = 1, 2, 3, 4, 5, 6
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
    for name in ("ntt_fwd", "ntt_inv", "bconv", "ks_rotate_hoisted", "ks_rotate_mac_hoisted", "ks_bsgs_linear_transform",
                 "hmult_relin_rescale", "hmult_relin_rescale_merged"):
        getattr(lib, name + "_u32").argtypes = getattr(lib, name).argtypes
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


# ---- size checks ----------------------------------------------------------------------------------------------------
# The C ABI takes bare pointers and cannot know how large the caller's tensors are; a tensor that is too small would
# make a kernel read or write outside its allocation (a GPU memory fault).  Every wrapper therefore checks element
# counts against what the header documents before anything is handed to the library.

def _batch_of(t: torch.Tensor, per_item: int, what: str) -> int:
    n = t.numel()
    if per_item <= 0 or n == 0 or n % per_item:
        raise KsError(f"{what}: {n} elements is not a positive multiple of {per_item} (one batch item)")
    return n // per_item


def _need(t: torch.Tensor, want: int, what: str, exact: bool = True) -> None:
    n = t.numel()
    if (n != want) if exact else (n < want):
        raise KsError(f"{what}: expected {'' if exact else 'at least '}{want} elements, got {n}")


def _level(ctx: Context, ell: int, lo: int = 1) -> None:
    if not (lo <= ell <= ctx.L):
        raise KsError(f"level {ell} outside {lo}..{ctx.L}")


def _key_words(ctx: Context) -> int:
    return ctx.dnum * 2 * (ctx.L + ctx.K) * ctx.N


def _on_device(ctx: Context, *tensors) -> None:
    for t in tensors:
        if t is not None and not (t.is_cuda and t.device.index == ctx.device):
            raise KsError(f"tensor on {t.device}, context on cuda:{ctx.device}")


def _ntt(name: str, dtype, ctx: Context, data: torch.Tensor, mod_ids) -> None:
    nl = len(mod_ids)
    batch = _batch_of(data, nl * ctx.N, f"{name} data")
    _on_device(ctx, data)
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(data, dtype), _u32_array(mod_ids), nl, batch, _stream()), name)


def ntt_fwd(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    """In place on data [batch][nlimbs][N]."""
    _ntt("ntt_fwd", torch.int64, ctx, data, mod_ids)


def ntt_inv(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    _ntt("ntt_inv", torch.int64, ctx, data, mod_ids)


def ntt_fwd_u32(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    """In place on an int32 tensor [batch][nlimbs][N] holding one residue (< 2^32) per 32-bit word."""
    _ntt("ntt_fwd_u32", torch.int32, ctx, data, mod_ids)


def ntt_inv_u32(ctx: Context, data: torch.Tensor, mod_ids) -> None:
    _ntt("ntt_inv_u32", torch.int32, ctx, data, mod_ids)


def bconv_prepare(ctx: Context, src_ids, dst_ids) -> None:
    """Set-up call: builds the constant table of this (source, target) list pair once; bconv needs it."""
    _check(load_library().bconv_prepare(ctx.handle, _u32_array(src_ids), len(src_ids), _u32_array(dst_ids), len(dst_ids)),
           "bconv_prepare")


def _bconv(name: str, dtype, ctx: Context, x: torch.Tensor, src_ids, out: torch.Tensor, dst_ids) -> None:
    batch = _batch_of(x, len(src_ids) * ctx.N, f"{name} input")
    _need(out, batch * len(dst_ids) * ctx.N, f"{name} output")
    _on_device(ctx, x, out)
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(x, dtype), _u32_array(src_ids), len(src_ids), _dev_ptr(out, dtype),
                                         _u32_array(dst_ids), len(dst_ids), batch, _stream()), name)


def bconv(ctx: Context, x: torch.Tensor, src_ids, out: torch.Tensor, dst_ids) -> None:
    _bconv("bconv", torch.int64, ctx, x, src_ids, out, dst_ids)


def bconv_u32(ctx: Context, x: torch.Tensor, src_ids, out: torch.Tensor, dst_ids) -> None:
    """bconv on int32 tensors holding one residue (< 2^32) per 32-bit word."""
    _bconv("bconv_u32", torch.int32, ctx, x, src_ids, out, dst_ids)


def _workspace_ok(ctx: Context, ws: torch.Tensor, op: int, ell: int, batch: int, n_rot: int = 0) -> None:
    if getattr(ctx, "handle", None) is not None:
        _need(ws, -(-ks_workspace_bytes(ctx, op, ell, batch, n_rot) // 8), "workspace", exact=False)


def ks_keyswitch(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor, ws: torch.Tensor) -> None:
    _level(ctx, ell)
    batch = _batch_of(d, ell * ctx.N, "ks_keyswitch d")
    _need(evk, _key_words(ctx), "evaluation key", exact=False)
    _need(out, batch * 2 * ell * ctx.N, "ks_keyswitch out")
    _workspace_ok(ctx, ws, KS_OP_KEYSWITCH, ell, batch)
    _on_device(ctx, d, evk, out, ws)
    _check(load_library().ks_keyswitch(ctx.handle, _dev_ptr(d), ell, _dev_ptr(evk), _dev_ptr(out), batch, _dev_ptr(ws),
                                       ws.numel() * 8, _stream()), "ks_keyswitch")


def ks_static_workspace_bytes() -> int:
    return int(load_library().ks_static_workspace_bytes())


def ks_keyswitch_static(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor) -> None:
    """ks_keyswitch on the library's own static scratch array: no workspace argument, no allocation."""
    _level(ctx, ell)
    batch = _batch_of(d, ell * ctx.N, "ks_keyswitch_static d")
    _need(evk, _key_words(ctx), "evaluation key", exact=False)
    _need(out, batch * 2 * ell * ctx.N, "ks_keyswitch_static out")
    _on_device(ctx, d, evk, out)
    _check(load_library().ks_keyswitch_static(ctx.handle, _dev_ptr(d), ell, _dev_ptr(evk), _dev_ptr(out), batch, _stream()),
           "ks_keyswitch_static")


def _rotation_args(ctx: Context, ct, ell, galois, rot_keys, what):
    _level(ctx, ell)
    batch = _batch_of(ct, 2 * ell * ctx.N, f"{what} ct")
    if len(galois) != len(rot_keys) or not rot_keys:
        raise KsError(f"{what}: {len(galois)} Galois elements for {len(rot_keys)} keys")
    for k in rot_keys:
        if k is not None:
            _need(k, _key_words(ctx), "rotation key", exact=False)
    return batch


def _rotate_hoisted(name, dtype, op, ctx, ct, ell, galois, rot_keys, out, ws) -> None:
    batch = _rotation_args(ctx, ct, ell, galois, rot_keys, name)
    if any(k is None for k in rot_keys):
        raise KsError(f"{name}: every rotation needs a key")
    _need(out, batch * len(rot_keys) * 2 * ell * ctx.N, f"{name} out")
    _workspace_ok(ctx, ws, op, ell, batch, len(rot_keys))
    _on_device(ctx, ct, out, ws, *rot_keys)
    ptrs = (_vp * len(rot_keys))(*[_dev_ptr(k, dtype) for k in rot_keys])
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(ct, dtype), ell, _u32_array(galois), ptrs, len(rot_keys),
                                         _dev_ptr(out, dtype), batch, _dev_ptr(ws), ws.numel() * 8, _stream()), name)


def ks_rotate_hoisted(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, out: torch.Tensor, ws: torch.Tensor) -> None:
    _rotate_hoisted("ks_rotate_hoisted", torch.int64, KS_OP_ROTATE_HOISTED, ctx, ct, ell, galois, rot_keys, out, ws)


def ks_rotate_hoisted_u32(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, out: torch.Tensor, ws: torch.Tensor) -> None:
    """ct, keys, out: int32 tensors, one residue (< 2^32) per word; ws: int64, sized for KS_OP_ROTATE_HOISTED_U32."""
    _rotate_hoisted("ks_rotate_hoisted_u32", torch.int32, KS_OP_ROTATE_HOISTED_U32, ctx, ct, ell, galois, rot_keys, out, ws)


def _hmult_args(ctx: Context, cta, ctb, ell, rlk, out, ws, what):
    _level(ctx, ell, 2)
    batch = _batch_of(cta, 2 * ell * ctx.N, f"{what} cta")
    _need(ctb, cta.numel(), f"{what} ctb")
    _need(rlk, _key_words(ctx), "relinearisation key", exact=False)
    _need(out, batch * 2 * (ell - 1) * ctx.N, f"{what} out")
    _workspace_ok(ctx, ws, KS_OP_HMULT_RELIN_RESCALE, ell, batch)
    _on_device(ctx, cta, ctb, rlk, out, ws)
    return batch


def _hmult(name, dtype, ctx, cta, ctb, ell, rlk, out, ws) -> None:
    batch = _hmult_args(ctx, cta, ctb, ell, rlk, out, ws, name)
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(cta, dtype), _dev_ptr(ctb, dtype), ell, _dev_ptr(rlk, dtype),
                                         _dev_ptr(out, dtype), batch, _dev_ptr(ws), ws.numel() * 8, _stream()), name)


def hmult_relin_rescale(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor, out: torch.Tensor,
                        ws: torch.Tensor) -> None:
    _hmult("hmult_relin_rescale", torch.int64, ctx, cta, ctb, ell, rlk, out, ws)


def hmult_relin_rescale_merged(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor, out: torch.Tensor,
                               ws: torch.Tensor) -> None:
    _hmult("hmult_relin_rescale_merged", torch.int64, ctx, cta, ctb, ell, rlk, out, ws)


def hmult_relin_rescale_u32(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor, out: torch.Tensor,
                            ws: torch.Tensor) -> None:
    """cta, ctb, rlk, out: int32 tensors, one residue (< 2^32) per word; ws: int64 as for hmult_relin_rescale."""
    _hmult("hmult_relin_rescale_u32", torch.int32, ctx, cta, ctb, ell, rlk, out, ws)


def hmult_relin_rescale_merged_u32(ctx: Context, cta: torch.Tensor, ctb: torch.Tensor, ell: int, rlk: torch.Tensor,
                                   out: torch.Tensor, ws: torch.Tensor) -> None:
    _hmult("hmult_relin_rescale_merged_u32", torch.int32, ctx, cta, ctb, ell, rlk, out, ws)


def _ptr_array(tensors, dtype=torch.int64):
    """Host array of device pointers; None entries become NULL."""
    return (_vp * len(tensors))(*[None if t is None else _dev_ptr(t, dtype) for t in tensors])


def _plaintexts_ok(ctx: Context, pts) -> None:
    for w in pts:
        if w is not None:
            _need(w, (ctx.L + ctx.K) * ctx.N, "plaintext", exact=False)


def _rotate_mac(name, dtype, op, ctx, ct, ell, galois, rot_keys, pts, out, ws) -> None:
    batch = _rotation_args(ctx, ct, ell, galois, rot_keys, name)
    if len(pts) != len(rot_keys):
        raise KsError(f"{name}: {len(pts)} plaintexts for {len(rot_keys)} rotations")
    _plaintexts_ok(ctx, pts)
    _need(out, batch * 2 * ell * ctx.N, f"{name} out")
    _workspace_ok(ctx, ws, op, ell, batch, len(rot_keys))
    _on_device(ctx, ct, out, ws, *rot_keys, *pts)
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(ct, dtype), ell, _u32_array(galois), _ptr_array(rot_keys, dtype),
                                         _ptr_array(pts, dtype), len(rot_keys), _dev_ptr(out, dtype), batch, _dev_ptr(ws),
                                         ws.numel() * 8, _stream()), name)


def ks_rotate_mac_hoisted(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, pts, out: torch.Tensor, ws: torch.Tensor) -> None:
    _rotate_mac("ks_rotate_mac_hoisted", torch.int64, KS_OP_ROTATE_HOISTED, ctx, ct, ell, galois, rot_keys, pts, out, ws)


def ks_rotate_mac_hoisted_u32(ctx: Context, ct: torch.Tensor, ell: int, galois, rot_keys, pts, out: torch.Tensor,
                              ws: torch.Tensor) -> None:
    """ct, keys, plaintexts, out: int32 tensors, one residue (< 2^32) per word; ws: int64, KS_OP_ROTATE_HOISTED_U32."""
    _rotate_mac("ks_rotate_mac_hoisted_u32", torch.int32, KS_OP_ROTATE_HOISTED_U32, ctx, ct, ell, galois, rot_keys, pts, out, ws)


def _bsgs(name, dtype, op, ctx, ct, ell, baby_galois, baby_keys, giant_galois, giant_keys, pts, out, ws) -> None:
    batch = _rotation_args(ctx, ct, ell, baby_galois, baby_keys, f"{name} (baby steps)")
    _rotation_args(ctx, ct, ell, giant_galois, giant_keys, f"{name} (giant steps)")
    if len(pts) != len(giant_keys) or any(len(row) != len(baby_keys) for row in pts):
        raise KsError(f"{name}: plaintexts must form n2 rows of n1 entries")
    flat = [w for row in pts for w in row]
    _plaintexts_ok(ctx, flat)
    _need(out, batch * 2 * ell * ctx.N, f"{name} out")
    _workspace_ok(ctx, ws, op, ell, batch)
    _on_device(ctx, ct, out, ws, *baby_keys, *giant_keys, *flat)
    _check(getattr(load_library(), name)(ctx.handle, _dev_ptr(ct, dtype), ell, _u32_array(baby_galois), _ptr_array(baby_keys, dtype),
                                         len(baby_keys), _u32_array(giant_galois), _ptr_array(giant_keys, dtype), len(giant_keys),
                                         _ptr_array(flat, dtype), _dev_ptr(out, dtype), batch, _dev_ptr(ws), ws.numel() * 8, _stream()),
           name)


def ks_bsgs_linear_transform(ctx: Context, ct: torch.Tensor, ell: int, baby_galois, baby_keys, giant_galois, giant_keys, pts,
                             out: torch.Tensor, ws: torch.Tensor) -> None:
    """pts: n2 rows of n1 plaintext tensors (or None)."""
    _bsgs("ks_bsgs_linear_transform", torch.int64, KS_OP_BSGS, ctx, ct, ell, baby_galois, baby_keys, giant_galois, giant_keys, pts,
          out, ws)


def ks_bsgs_linear_transform_u32(ctx: Context, ct: torch.Tensor, ell: int, baby_galois, baby_keys, giant_galois, giant_keys, pts,
                                 out: torch.Tensor, ws: torch.Tensor) -> None:
    """ct, keys, plaintexts, out: int32 tensors, one residue (< 2^32) per word; ws: int64, sized for KS_OP_BSGS_U32."""
    _bsgs("ks_bsgs_linear_transform_u32", torch.int32, KS_OP_BSGS_U32, ctx, ct, ell, baby_galois, baby_keys, giant_galois,
          giant_keys, pts, out, ws)


def ks_keyswitch_u32(ctx: Context, d: torch.Tensor, ell: int, evk: torch.Tensor, out: torch.Tensor, ws: torch.Tensor) -> None:
    """d, evk, out: int32 tensors holding one residue (< 2^32) per 32-bit word; ws as for ks_keyswitch (int64)."""
    _level(ctx, ell)
    batch = _batch_of(d, ell * ctx.N, "ks_keyswitch_u32 d")
    _need(evk, _key_words(ctx), "evaluation key", exact=False)
    _need(out, batch * 2 * ell * ctx.N, "ks_keyswitch_u32 out")
    _workspace_ok(ctx, ws, KS_OP_KEYSWITCH, ell, batch)
    _on_device(ctx, d, evk, out, ws)
    _check(load_library().ks_keyswitch_u32(ctx.handle, _dev_ptr(d, torch.int32), ell, _dev_ptr(evk, torch.int32),
                                           _dev_ptr(out, torch.int32), batch, _dev_ptr(ws), ws.numel() * 8, _stream()), "ks_keyswitch_u32")
