"""ctypes wrapper around the plain-C reference tier (ks_oracle.c).  TEST INFRASTRUCTURE ONLY.

All arrays are numpy uint64, C-contiguous, host memory; layouts are those documented in
ks_oracle.c.  `build()` compiles the C file with gcc; nothing here touches the GPU library.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ks_oracle.c")
_LIB = os.path.join(_HERE, "libks_oracle.so")
_lib = None

_u64p = ctypes.POINTER(ctypes.c_uint64)
_u32p = ctypes.POINTER(ctypes.c_uint32)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_create.restype = ctypes.c_void_p
        lib.orc_create.argtypes = [ctypes.c_int] * 4 + [_u64p] * 3
        lib.orc_destroy.argtypes = [ctypes.c_void_p]
        lib.orc_ntt_fwd.argtypes = [ctypes.c_void_p, _u64p, _u32p, ctypes.c_int, ctypes.c_int]
        lib.orc_ntt_inv.argtypes = [ctypes.c_void_p, _u64p, _u32p, ctypes.c_int, ctypes.c_int]
        lib.orc_bconv.argtypes = [ctypes.c_void_p, _u64p, _u32p, ctypes.c_int, _u64p, _u32p, ctypes.c_int, ctypes.c_int]
        lib.orc_keyswitch.argtypes = [ctypes.c_void_p, _u64p, ctypes.c_int, _u64p, _u64p, ctypes.c_int]
        lib.orc_rotate_hoisted.argtypes = [ctypes.c_void_p, _u64p, ctypes.c_int, _u32p,
                                           ctypes.POINTER(_u64p), ctypes.c_int, _u64p, ctypes.c_int]
        lib.orc_rotate_mac_hoisted.argtypes = [ctypes.c_void_p, _u64p, ctypes.c_int, _u32p, ctypes.POINTER(_u64p),
                                               ctypes.POINTER(_u64p), ctypes.c_int, _u64p, ctypes.c_int]
        lib.orc_bsgs_linear_transform.argtypes = [ctypes.c_void_p, _u64p, ctypes.c_int, _u32p, ctypes.POINTER(_u64p), ctypes.c_int,
                                                  _u32p, ctypes.POINTER(_u64p), ctypes.c_int, ctypes.POINTER(_u64p), _u64p,
                                                  ctypes.c_int]
        lib.orc_hmult_relin_rescale.argtypes = [ctypes.c_void_p, _u64p, _u64p, ctypes.c_int, _u64p, _u64p, ctypes.c_int]
        lib.orc_hmult_relin_rescale_merged.argtypes = [ctypes.c_void_p, _u64p, _u64p, ctypes.c_int, _u64p, _u64p, ctypes.c_int]
        lib.orc_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p64(a: np.ndarray):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_u64p)


def _ptr_array(arrays):
    """Array of limb pointers for a list of uint64 arrays; None entries become NULL."""
    return (_u64p * len(arrays))(*[_u64p() if a is None else _p64(a) for a in arrays])


def _p32(a: np.ndarray):
    assert a.dtype == np.uint32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_u32p)


def max_threads() -> int:
    return int(_load().orc_max_threads())


class COracle:
    """Holds the per-modulus power tables for one parameter set."""

    def __init__(self, logN: int, q, p, dnum: int, psi):
        lib = _load()
        self.logN, self.N = logN, 1 << logN
        self.L, self.K, self.dnum = len(q), len(p), dnum
        qa = np.asarray(list(q), dtype=np.uint64)
        pa = np.asarray(list(p) if len(p) else [0], dtype=np.uint64)
        sa = np.asarray(list(psi), dtype=np.uint64)
        assert len(sa) == self.L + self.K
        self._h = lib.orc_create(logN, self.L, self.K, dnum, _p64(qa), _p64(pa), _p64(sa))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.orc_destroy(self._h)
            self._h = None

    def ntt_fwd(self, data: np.ndarray, mod_ids) -> np.ndarray:
        """data [batch][nlimbs][N] -> transformed copy."""
        out = np.ascontiguousarray(data, dtype=np.uint64).copy()
        ids = np.asarray(mod_ids, dtype=np.uint32)
        batch = out.size // (len(ids) * self.N)
        _load().orc_ntt_fwd(self._h, _p64(out), _p32(ids), len(ids), batch)
        return out

    def ntt_inv(self, data: np.ndarray, mod_ids) -> np.ndarray:
        out = np.ascontiguousarray(data, dtype=np.uint64).copy()
        ids = np.asarray(mod_ids, dtype=np.uint32)
        batch = out.size // (len(ids) * self.N)
        _load().orc_ntt_inv(self._h, _p64(out), _p32(ids), len(ids), batch)
        return out

    def bconv(self, x: np.ndarray, src_ids, dst_ids) -> np.ndarray:
        """x [batch][n_src][N] coefficient domain -> [batch][n_dst][N]."""
        x = np.ascontiguousarray(x, dtype=np.uint64)
        src = np.asarray(src_ids, dtype=np.uint32)
        dst = np.asarray(dst_ids, dtype=np.uint32)
        batch = x.size // (len(src) * self.N)
        out = np.zeros((batch, len(dst), self.N), dtype=np.uint64)
        _load().orc_bconv(self._h, _p64(x), _p32(src), len(src), _p64(out), _p32(dst), len(dst), batch)
        return out

    def keyswitch(self, d: np.ndarray, evk: np.ndarray, ell: int | None = None) -> np.ndarray:
        """d [batch][ell][N], evk [dnum][2][L+K][N] -> [batch][2][ell][N]."""
        ell = self.L if ell is None else ell
        d = np.ascontiguousarray(d, dtype=np.uint64)
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        batch = d.size // (ell * self.N)
        out = np.zeros((batch, 2, ell, self.N), dtype=np.uint64)
        _load().orc_keyswitch(self._h, _p64(d), ell, _p64(evk), _p64(out), batch)
        return out

    def rotate_hoisted(self, ct: np.ndarray, galois, rot_keys, ell: int | None = None) -> np.ndarray:
        """ct [batch][2][ell][N]; rot_keys: list of [dnum][2][L+K][N] -> [batch][n_rot][2][ell][N]."""
        ell = self.L if ell is None else ell
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        keys = [np.ascontiguousarray(k, dtype=np.uint64) for k in rot_keys]
        g = np.asarray(galois, dtype=np.uint32)
        batch = ct.size // (2 * ell * self.N)
        out = np.zeros((batch, len(g), 2, ell, self.N), dtype=np.uint64)
        ptrs = (_u64p * len(keys))(*[_p64(k) for k in keys])
        _load().orc_rotate_hoisted(self._h, _p64(ct), ell, _p32(g), ptrs, len(g), _p64(out), batch)
        return out

    def rotate_mac_hoisted(self, ct: np.ndarray, galois, rot_keys, pts, ell: int | None = None) -> np.ndarray:
        """ct [batch][2][ell][N]; rot_keys: list of [dnum][2][L+K][N]; pts: list of [L+K][N] -> [batch][2][ell][N]."""
        ell = self.L if ell is None else ell
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        keys = [None if k is None else np.ascontiguousarray(k, dtype=np.uint64) for k in rot_keys]
        pls = [None if w is None else np.ascontiguousarray(w, dtype=np.uint64) for w in pts]
        g = np.asarray(galois, dtype=np.uint32)
        batch = ct.size // (2 * ell * self.N)
        out = np.zeros((batch, 2, ell, self.N), dtype=np.uint64)
        kp = _ptr_array(keys)
        pp = _ptr_array(pls)
        _load().orc_rotate_mac_hoisted(self._h, _p64(ct), ell, _p32(g), kp, pp, len(g), _p64(out), batch)
        return out

    def bsgs_linear_transform(self, ct: np.ndarray, baby_galois, baby_keys, giant_galois, giant_keys, pts,
                              ell: int | None = None) -> np.ndarray:
        """ct [batch][2][ell][N]; keys: lists of [dnum][2][L+K][N] (None where the Galois element is 1);
        pts[g][b]: [L+K][N] or None (= 1) -> [batch][2][ell][N]."""
        ell = self.L if ell is None else ell
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        cont = lambda x: None if x is None else np.ascontiguousarray(x, dtype=np.uint64)
        bk, gk = [cont(k) for k in baby_keys], [cont(k) for k in giant_keys]
        flat = [cont(w) for row in pts for w in row]
        bg, gg = np.asarray(baby_galois, dtype=np.uint32), np.asarray(giant_galois, dtype=np.uint32)
        batch = ct.size // (2 * ell * self.N)
        out = np.zeros((batch, 2, ell, self.N), dtype=np.uint64)
        _load().orc_bsgs_linear_transform(self._h, _p64(ct), ell, _p32(bg), _ptr_array(bk), len(bg), _p32(gg), _ptr_array(gk),
                                          len(gg), _ptr_array(flat), _p64(out), batch)
        return out

    def hmult_relin_rescale(self, cta: np.ndarray, ctb: np.ndarray, rlk: np.ndarray, ell: int | None = None) -> np.ndarray:
        """cta, ctb [batch][2][ell][N] -> [batch][2][ell-1][N]."""
        ell = self.L if ell is None else ell
        cta = np.ascontiguousarray(cta, dtype=np.uint64)
        ctb = np.ascontiguousarray(ctb, dtype=np.uint64)
        rlk = np.ascontiguousarray(rlk, dtype=np.uint64)
        batch = cta.size // (2 * ell * self.N)
        out = np.zeros((batch, 2, ell - 1, self.N), dtype=np.uint64)
        _load().orc_hmult_relin_rescale(self._h, _p64(cta), _p64(ctb), ell, _p64(rlk), _p64(out), batch)
        return out

    def hmult_relin_rescale_merged(self, cta: np.ndarray, ctb: np.ndarray, rlk: np.ndarray, ell: int | None = None) -> np.ndarray:
        """As hmult_relin_rescale, with ModDown and rescale merged into one division by P q_{ell-1}."""
        ell = self.L if ell is None else ell
        cta = np.ascontiguousarray(cta, dtype=np.uint64)
        ctb = np.ascontiguousarray(ctb, dtype=np.uint64)
        rlk = np.ascontiguousarray(rlk, dtype=np.uint64)
        batch = cta.size // (2 * ell * self.N)
        out = np.zeros((batch, 2, ell - 1, self.N), dtype=np.uint64)
        _load().orc_hmult_relin_rescale_merged(self._h, _p64(cta), _p64(ctb), ell, _p64(rlk), _p64(out), batch)
        return out
