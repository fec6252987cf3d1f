"""Position-weighted 64-bit checksums of residue tensors (test infrastructure).

Two independent weighted sums modulo 2^64 over the flattened tensor; int64 arithmetic wraps, integer addition is
associative, so the value is the same on the CPU and on the GPU whatever the reduction order.  Used to compare whole
full-size outputs against values the CPU reference produced ahead of time (tests/golden/fullsize_checksums.txt)."""

import torch


def _s64(x: int) -> int:
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_A = _s64(0x9E3779B97F4A7C15)
_B = _s64(0xC2B2AE3D27D4EB4F)


def checksum(t: torch.Tensor) -> tuple[int, int]:
    """t: int64 tensor (any shape, CPU or CUDA).  Returns two unsigned 64-bit integers."""
    x = t.reshape(-1)
    i = torch.arange(x.numel(), dtype=torch.int64, device=x.device)
    w1 = (2 * i + 1) * _A
    j = i ^ ((i >> 7) & ((1 << 57) - 1))
    w2 = (j * _B) | 1
    c1 = int((x * w1).sum().item()) & ((1 << 64) - 1)
    c2 = int((x * w2).sum().item()) & ((1 << 64) - 1)
    return c1, c2
