"""Seeded synthetic inputs for the key-switching workloads.

This module serves both the CPU reference and the GPU library and therefore holds none of the
method's arithmetic: it only picks moduli, draws pseudo-random residues / secrets / errors and
names the workload shapes.  Residues come from a counter-based mixer, so any slab of a large
tensor can be regenerated on its own, on the CPU or directly in GPU memory, bit-identically.
"""

from __future__ import annotations

import numpy as np
import torch

# --------------------------------------------------------------------------------------
# workload shapes (ring degree, ciphertext primes L, special primes K, digits, batch ...)
# --------------------------------------------------------------------------------------

CONFIGS = {
    1: dict(name="tiny-keyswitch", logN=12, L=4, K=2, dnum=2, batch=1, seed=1001),
    2: dict(name="bootstrap-keyswitch", logN=16, L=24, K=8, dnum=3, batch=1, seed=1002),
    3: dict(name="hoisted-rotations", logN=16, L=24, K=8, dnum=3, batch=64, n_rot=16, seed=1003),
    4: dict(name="batched-ntt", logN=16, L=60, K=0, dnum=1, batch=32, seed=1004),
    5: dict(name="hmult-relin-rescale", logN=16, L=35, K=12, dnum=3, batch=256, seed=1005),
}


def _is_prime(n: int) -> bool:
    if n < 2:
        return False
    for p in (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37):
        if n % p == 0:
            return n == p
    d, s = n - 1, 0
    while d % 2 == 0:
        d, s = d // 2, s + 1
    for a in (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37):
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(s - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def prime_list(logN: int, count: int, bits: int = 36) -> list[int]:
    """Largest `count` primes below 2^bits congruent to 1 modulo 2N, descending."""
    step = 2 << logN
    m = (1 << bits) + 1 - step
    out = []
    while len(out) < count:
        if _is_prime(m):
            out.append(m)
        m -= step
    return out


def moduli(cfg: dict) -> tuple[list[int], list[int]]:
    """(q, p): special primes take the K largest primes, ciphertext primes the next L."""
    pl = prime_list(cfg["logN"], cfg["L"] + cfg["K"], cfg.get("bits", 36))
    return pl[cfg["K"]:], pl[:cfg["K"]]


def galois_elements(logN: int, n_rot: int) -> list[int]:
    """g_r = 5^r mod 2N for r = 1..n_rot."""
    return [pow(5, r, 2 << logN) for r in range(1, n_rot + 1)]


# --------------------------------------------------------------------------------------
# counter-based uniform residues
# --------------------------------------------------------------------------------------

def _s64(x: int) -> int:
    """Wrap an unsigned 64-bit constant into the signed range torch.int64 holds."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_TENSOR = _s64(0xD1B54A32D192ED03)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift on int64 storage."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    """SplitMix64 output function; int64 multiplication wraps modulo 2^64."""
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def uniform_slab(seed: int, tensor_id: int, slab_index: int, mods: list[int], N: int,
                 device="cpu") -> torch.Tensor:
    """Slab `slab_index` of tensor `tensor_id`: shape [len(mods)][N], int64, residue of limb i in [0, mods[i]).

    Element at flat position f of the whole tensor is (mix64(key + f) >> 28) mod m, i.e. a
    36-bit word reduced by the limb's modulus."""
    nl = len(mods)
    base = slab_index * nl * N
    idx = torch.arange(base, base + nl * N, dtype=torch.int64, device=device).view(nl, N)
    key = _s64(seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03)
    z = _mix64(idx + key)
    word = _lsr(z, 28)
    m = torch.tensor(mods, dtype=torch.int64, device=device).view(nl, 1)
    return word % m


def uniform_residues(seed: int, tensor_id: int, lead: tuple[int, ...], mods: list[int], N: int,
                     device="cpu") -> torch.Tensor:
    """Tensor [*lead][len(mods)][N] of uniform residues, generated slab by slab."""
    n_slabs = int(np.prod(lead)) if len(lead) else 1
    out = torch.empty((n_slabs, len(mods), N), dtype=torch.int64, device=device)
    for s in range(n_slabs):
        out[s] = uniform_slab(seed, tensor_id, s, mods, N, device)
    return out.view(*lead, len(mods), N)


def as_u64(t: torch.Tensor) -> np.ndarray:
    """Host numpy uint64 view of an int64 tensor (copying it to the host first if needed)."""
    return t.detach().cpu().contiguous().numpy().view(np.uint64)


# --------------------------------------------------------------------------------------
# secrets and errors for the small configuration with real keys
# --------------------------------------------------------------------------------------

def ternary_secret(seed: int, N: int) -> list[int]:
    """Coefficients uniform in {-1, 0, 1}."""
    rng = np.random.RandomState(seed)
    return [int(x) - 1 for x in rng.randint(0, 3, size=N)]


def gaussian_error(seed: int, N: int, sigma: float = 3.2, bound: int = 19) -> list[int]:
    """Rounded Gaussian with standard deviation sigma, truncated to |e| <= bound."""
    rng = np.random.RandomState(seed)
    e = np.rint(rng.normal(0.0, sigma, size=N)).astype(np.int64)
    return [int(x) for x in np.clip(e, -bound, bound)]
