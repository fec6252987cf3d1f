#!/usr/bin/env python3
"""Writes tests/golden/fullsize_checksums.txt: checksums (tests/checksum.py) of the CPU reference's outputs for the full-size
workloads whose results are too large to recompute inside a GPU test run -- configuration 3 (64 ciphertexts x 16 hoisted
rotations) and configuration 5 (256 multiplications, both variants).  Calls only ks_inputs (seeded inputs) and oracle/.
Takes several minutes of CPU time; run from the repository root:  python tests/golden/make_fullsize_checksums.py"""

import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import ks_inputs                      # noqa: E402
from checksum import checksum         # noqa: E402
from oracle import c_tier             # noqa: E402
from oracle import ckks_ref as R      # noqa: E402


def as_t(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64))


def u64(t: torch.Tensor) -> np.ndarray:
    return t.numpy().view(np.uint64)


def main():
    c_tier.build()
    lines = ["# workload item... checksum1 checksum2 (hex); written by tests/golden/make_fullsize_checksums.py"]
    t0 = time.time()

    cfg = ks_inputs.CONFIGS[3]
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, nrot, dnum, seed = cfg["logN"], cfg["L"], cfg["batch"], cfg["n_rot"], cfg["dnum"], cfg["seed"]
    N = 1 << logN
    ref = c_tier.COracle(logN, q, p, dnum, [R.minimal_psi(m, logN) for m in q + p])
    keys = [u64(ks_inputs.uniform_residues(seed, 10 + r, (dnum, 2), q + p, N)) for r in range(nrot)]
    gal = ks_inputs.galois_elements(logN, nrot)
    for b in range(B):
        ct = np.stack([u64(ks_inputs.uniform_slab(seed, 1, 2 * b + c, q, N)) for c in range(2)])[None]
        out = ref.rotate_hoisted(ct, gal, keys, L)          # [1][nrot][2][L][N]
        for r in range(nrot):
            c1, c2 = checksum(as_t(out[0, r]))
            lines.append(f"cfg3_rotate {b} {r} {c1:016x} {c2:016x}")
        print(f"cfg3 ciphertext {b + 1}/{B}  {time.time() - t0:.0f} s", flush=True)
    del keys

    cfg = ks_inputs.CONFIGS[5]
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, dnum, seed = cfg["logN"], cfg["L"], cfg["batch"], cfg["dnum"], cfg["seed"]
    ref = c_tier.COracle(logN, q, p, dnum, [R.minimal_psi(m, logN) for m in q + p])
    rlk = u64(ks_inputs.uniform_residues(seed, 3, (dnum, 2), q + p, N))
    for b in range(B):
        cta = np.stack([u64(ks_inputs.uniform_slab(seed, 1, 2 * b + c, q, N)) for c in range(2)])[None]
        ctb = np.stack([u64(ks_inputs.uniform_slab(seed, 2, 2 * b + c, q, N)) for c in range(2)])[None]
        for name, fn in (("cfg5_hmult", ref.hmult_relin_rescale), ("cfg5_hmult_merged", ref.hmult_relin_rescale_merged)):
            c1, c2 = checksum(as_t(fn(cta, ctb, rlk, L)[0]))
            lines.append(f"{name} {b} 0 {c1:016x} {c2:016x}")
        if (b + 1) % 16 == 0:
            print(f"cfg5 pair {b + 1}/{B}  {time.time() - t0:.0f} s", flush=True)

    path = os.path.join(ROOT, "tests", "golden", "fullsize_checksums.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", path, len(lines) - 1, "records")


if __name__ == "__main__":
    main()
