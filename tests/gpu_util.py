"""Helpers shared by the GPU parity tests: build a library context and a C-reference context for the
same parameters, and move seeded inputs between torch (device) and numpy (host)."""

import numpy as np
import torch

import ks_inputs
import paper_2512_11269_amd as K
from oracle import c_tier
from oracle import ckks_ref as R


class Setup:
    def __init__(self, logN, L, Kk, dnum, bits=36):
        cfg = dict(logN=logN, L=L, K=Kk, bits=bits)
        self.q, self.p = ks_inputs.moduli(cfg)
        self.logN, self.N, self.L, self.K, self.dnum = logN, 1 << logN, L, Kk, dnum
        self.moduli = self.q + self.p
        self.ctx = K.Context(logN, self.q, self.p, dnum)                    # library picks its own minimal psi
        psi = [R.minimal_psi(m, logN) for m in self.moduli]                 # reference picks its own
        self.ref = c_tier.COracle(logN, self.q, self.p, dnum, psi)

    def uniform(self, seed, tid, lead, ids):
        return ks_inputs.uniform_residues(seed, tid, lead, [self.moduli[m] for m in ids], self.N, device="cuda")


def host(t: torch.Tensor) -> np.ndarray:
    return ks_inputs.as_u64(t)


def workspace(ctx, op, ell, batch, n_rot=0):
    nbytes = K.ks_workspace_bytes(ctx, op, ell, batch, n_rot)
    assert nbytes > 0
    return torch.empty(nbytes // 8, dtype=torch.int64, device="cuda")


def assert_equal(got: torch.Tensor, want: np.ndarray):
    g = host(got).reshape(want.shape)
    if not np.array_equal(g, want):
        bad = np.argwhere(g != want)
        raise AssertionError(f"{len(bad)} of {want.size} residues differ; first at {bad[0].tolist()}: "
                             f"got {g[tuple(bad[0])]} want {want[tuple(bad[0])]}")
