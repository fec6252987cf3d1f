"""The plain-C reference under AddressSanitizer and UndefinedBehaviourSanitizer (host code only, no GPU): a driver that
includes oracle/ks_oracle.c calls every entry point at every level of two small parameter sets; the run must finish
clean.  The reference is the yardstick of every parity test, so it should not be reading a stray word itself."""

import os
import shutil
import subprocess

import pytest

import ks_inputs
from oracle import ckks_ref as R

HERE = os.path.dirname(os.path.abspath(__file__))
DRIVER = os.path.join(HERE, "sanitize", "oracle_driver.c")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if not shutil.which("gcc"):
        pytest.skip("gcc not available")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", DRIVER, "-o", exe, "-lm"])
    return exe


@pytest.mark.parametrize("logN,L,K,dnum", [(12, 4, 2, 2), (12, 5, 3, 3)])
def test_reference_runs_clean_under_sanitizers(driver, logN, L, K, dnum):
    q, p = ks_inputs.moduli(dict(logN=logN, L=L, K=K, bits=36))
    psi = [R.minimal_psi(m, logN) for m in q + p]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)
    out = subprocess.run([driver, str(logN), str(L), str(K), str(dnum)] + [str(v) for v in q + p + psi], capture_output=True,
                         text=True, timeout=600, env=env)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert out.stdout.strip().endswith("OK")
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr
