"""Pins for the pure-Python reference tier: every function is checked against something that is
not itself (brute force, big-integer CRT, closed forms, the decrypt-within-noise bound)."""

import os
import random

import pytest
import sympy

import ks_inputs
from oracle import ckks_ref as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "params.txt")


def _golden():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ------------------------------------------------------------------ parameters

def test_primes_match_golden_and_sympy():
    p12 = R.ntt_primes(12, 6)
    p16 = R.ntt_primes(16, 60)
    for kind, a, b in _golden():
        if kind == "primes12":
            assert p12[int(a)] == int(b)
        if kind == "primes16":
            assert p16[int(a)] == int(b)
    for logN, plist in ((12, p12), (16, p16)):
        step = 2 << logN
        assert plist == sorted(plist, reverse=True)
        assert all(p < 2 ** 36 and p.bit_length() == 36 and p % step == 1 and sympy.isprime(p) for p in plist)
        # nothing was skipped: every candidate between the top and the last one is composite unless listed
        cand = 2 ** 36 + 1 - step
        seen = []
        while cand >= plist[-1]:
            if sympy.isprime(cand):
                seen.append(cand)
            cand -= step
        assert seen == plist
    # the input generator's independent prime search agrees
    assert ks_inputs.prime_list(12, 6) == p12
    assert ks_inputs.prime_list(16, 60) == p16


def test_minimal_psi_golden_and_bruteforce():
    for kind, m, psi in _golden():
        if kind.startswith("psi"):
            logN = int(kind[3:])
            m, psi = int(m), int(psi)
            assert R.minimal_psi(m, logN) == psi
            assert pow(psi, 1 << logN, m) == m - 1
    # minimality by brute force over a small field: 12289 = 1 (mod 2^12)
    for logN in (3, 5, 11):
        m = 12289
        psi = R.minimal_psi(m, logN)
        brute = next(x for x in range(2, m) if pow(x, 1 << logN, m) == m - 1)
        assert psi == brute


def test_brv():
    assert [R.brv(k, 3) for k in range(8)] == [0, 4, 2, 6, 1, 5, 3, 7]
    assert all(R.brv(R.brv(k, 10), 10) == k for k in range(1024))


# ------------------------------------------------------------------ transform

@pytest.mark.parametrize("logN", [1, 2, 3, 5, 7])
def test_ntt_iterative_equals_definition(logN):
    rng = random.Random(logN)
    m = R.ntt_primes(logN, 2)[1]
    psi = R.minimal_psi(m, logN)
    a = [rng.randrange(m) for _ in range(1 << logN)]
    A = R.ntt_def(a, m, psi)
    assert R.ntt(a, m, psi) == A
    assert R.intt_def(A, m, psi) == a
    assert R.intt(A, m, psi) == a


def test_ntt_of_delta_and_X():
    logN, N = 6, 64
    m = R.ntt_primes(logN, 1)[0]
    psi = R.minimal_psi(m, logN)
    delta = [1] + [0] * (N - 1)
    assert R.ntt(delta, m, psi) == [1] * N
    X = [0, 1] + [0] * (N - 2)
    assert R.ntt(X, m, psi) == [pow(psi, 2 * R.brv(k, logN) + 1, m) for k in range(N)]


@pytest.mark.parametrize("logN", [3, 6, 8])
def test_convolution_theorem_vs_schoolbook(logN):
    rng = random.Random(100 + logN)
    N = 1 << logN
    m = R.ntt_primes(logN, 3)[2]
    psi = R.minimal_psi(m, logN)
    a = [rng.randrange(m) for _ in range(N)]
    b = [rng.randrange(m) for _ in range(N)]
    prod = [x * y % m for x, y in zip(R.ntt(a, m, psi), R.ntt(b, m, psi))]
    assert R.intt(prod, m, psi) == R.negacyclic_mul(a, b, m)


def test_negacyclic_wraparound_sign():
    # X^(N-1) * X = X^N = -1
    N, m = 8, 97
    a = [0] * N
    a[N - 1] = 1
    b = [0, 1] + [0] * (N - 2)
    assert R.negacyclic_mul(a, b, m) == [m - 1] + [0] * (N - 1)


@pytest.mark.parametrize("g", [1, 3, 5, 25, 127])
def test_automorphism_eval_is_coefficient_automorphism(g):
    logN, N = 6, 64
    rng = random.Random(g)
    m = R.ntt_primes(logN, 1)[0]
    psi = R.minimal_psi(m, logN)
    a = [rng.randrange(m) for _ in range(N)]
    via_coeff = R.ntt(R.automorphism_coeff(a, g, m), m, psi)
    assert R.automorphism_eval(R.ntt(a, m, psi), g) == via_coeff
    # definition check: sigma_g(a)(x) = a(x^g) at x = psi
    x = psi
    lhs = sum(c * pow(x, i, m) for i, c in enumerate(R.automorphism_coeff(a, g, m))) % m
    rhs = sum(c * pow(x, g * i, m) for i, c in enumerate(a)) % m
    assert lhs == rhs


# ------------------------------------------------------------------ base conversion

def test_bconv_crt_invariants():
    rng = random.Random(7)
    primes = R.ntt_primes(4, 7)
    src, dst = primes[:4], primes[4:]
    D = 1
    for q in src:
        D *= q
    N = 16
    values = [rng.randrange(D) for _ in range(N - 3)] + [0, 1, D - 1]
    limbs = [[v % q for v in values] for q in src]
    fast = R.bconv_fast(limbs, src, dst)
    exact = R.bconv_exact(limbs, src, dst)
    for n, v in enumerate(values):
        lifted = R.bconv_lift([limb[n] for limb in limbs], src)
        assert all(lifted % q == v % q for q in src)           # congruent to every source residue
        u, rem = divmod(lifted - v, D)
        assert rem == 0 and 0 <= u < len(src)                    # x + u D with 0 <= u < alpha
        assert R.crt_reconstruct([limb[n] for limb in limbs], src) == v
        for ti, t in enumerate(dst):
            assert exact[ti][n] == v % t
            assert (fast[ti][n] - exact[ti][n]) % t == u * D % t
    zero = [[0] * N for _ in src]
    assert R.bconv_fast(zero, src, dst) == [[0] * N for _ in dst]


def test_bconv_single_source_is_plain_reduction():
    rng = random.Random(8)
    primes = R.ntt_primes(4, 4)
    src, dst = primes[3:4], primes[:3]       # smallest prime as the source: x < q means x mod t = x
    x = [rng.randrange(src[0]) for _ in range(16)]
    assert R.bconv_fast([x], src, dst) == [[v % t for v in x] for t in dst]


# ------------------------------------------------------------------ key switching

def _small_params(logN=5, L=4, K=2, dnum=2):
    pl = R.ntt_primes(logN, L + K)
    return R.Params(logN, pl[K:], pl[:K], dnum)


def _uniform_poly(rng, pr, ids):
    return [[rng.randrange(pr.moduli[m]) for _ in range(pr.N)] for m in ids]


def _keys(pr, seed, s_from_signed, s_signed):
    rng = random.Random(seed)
    all_ids = list(range(pr.L + pr.K))
    ndig = len(pr.digits(pr.L))
    a = [_uniform_poly(rng, pr, all_ids) for _ in range(ndig)]
    e = [ks_inputs.gaussian_error(seed + 10 + j, pr.N) for j in range(ndig)]
    return R.switching_key(pr, R.to_eval(pr, s_from_signed, all_ids), R.to_eval(pr, s_signed, all_ids), a, e)


def _noise_bound(pr, ell):
    return pr.N * 19 * pr.L + pr.K * (pr.N + 1)


@pytest.mark.parametrize("L,K,dnum", [(4, 2, 2), (5, 2, 3), (3, 3, 1)])
def test_transparent_key_gives_exact_product(L, K, dnum):
    """With a_j = 0, e_j = 0 the switching key is b_j = [m in digit j] P s'; the pipeline must then
    return exactly (d s' mod Q, 0): checks decompose + raise + inner product + divide against
    schoolbook multiplication alone."""
    pr = _small_params(5, L, K, dnum)
    rng = random.Random(L * 100 + K * 10 + dnum)
    all_ids = list(range(pr.L + pr.K))
    ndig = len(pr.digits(pr.L))
    s_from = ks_inputs.ternary_secret(5, pr.N)
    zero_a = [[[0] * pr.N for _ in all_ids] for _ in range(ndig)]
    zero_e = [[0] * pr.N for _ in range(ndig)]
    s_from_eval = R.to_eval(pr, s_from, all_ids)
    evk = R.switching_key(pr, s_from_eval, s_from_eval, zero_a, zero_e)
    d = _uniform_poly(rng, pr, range(pr.L))
    o0, o1 = R.keyswitch(pr, d, evk)
    for i in range(pr.L):
        qi = pr.q[i]
        want = R.negacyclic_mul(R.intt(d[i], qi, pr.psi[i]), [x % qi for x in s_from], qi)
        assert R.intt(o0[i], qi, pr.psi[i]) == want
        assert o1[i] == [0] * pr.N


@pytest.mark.parametrize("L,K,dnum,ell", [(4, 2, 2, 4), (5, 2, 3, 5), (6, 3, 2, 4)])
def test_keyswitch_decrypts_within_noise_bound(L, K, dnum, ell):
    pr = _small_params(5, L, K, dnum)
    rng = random.Random(42 + L)
    s = ks_inputs.ternary_secret(1, pr.N)
    s_from = ks_inputs.ternary_secret(2, pr.N)
    evk = _keys(pr, 77, s_from, s)
    d = _uniform_poly(rng, pr, range(ell))
    o0, o1 = R.keyswitch(pr, d, evk, ell)
    s_eval = R.to_eval(pr, s, list(range(ell)))
    got = R.phase(pr, o0, o1, s_eval, ell)
    # target: d * s_from mod Q_ell, centred
    sf_eval = R.to_eval(pr, s_from, list(range(ell)))
    want_eval = [[x * y % pr.q[i] for x, y in zip(d[i], sf_eval[i])] for i in range(ell)]
    want = R.poly_to_big(pr, want_eval, ell)
    Q = pr.Q(ell)
    err = max(abs(((g - w + Q // 2) % Q) - Q // 2) for g, w in zip(got, want))
    assert err <= _noise_bound(pr, ell)
    assert err > 0          # a real key does add noise; zero would mean the error term was dropped


def test_keyswitch_cfg1_noise_bound():
    """Configuration 1 at full size (N = 2^12, L = 4, K = 2, dnum = 2) with a real relinearisation key."""
    cfg = ks_inputs.CONFIGS[1]
    q, p = ks_inputs.moduli(cfg)
    pr = R.Params(cfg["logN"], q, p, cfg["dnum"])
    assert pr.q == R.ntt_primes(12, 6)[2:] and pr.p == R.ntt_primes(12, 6)[:2]
    s = ks_inputs.ternary_secret(cfg["seed"], pr.N)
    all_ids = list(range(pr.L + pr.K))
    s_eval = R.to_eval(pr, s, all_ids)
    s2_eval = [[x * x % pr.moduli[m] for x in s_eval[m]] for m in all_ids]
    a = [[[int(v) for v in row] for row in ks_inputs.uniform_slab(cfg["seed"], 10 + j, 0, pr.moduli, pr.N).tolist()]
         for j in range(pr.dnum)]
    e = [ks_inputs.gaussian_error(cfg["seed"] + 1 + j, pr.N) for j in range(pr.dnum)]
    evk = R.switching_key(pr, s2_eval, s_eval, a, e)
    d = [[int(v) for v in row] for row in ks_inputs.uniform_slab(cfg["seed"], 1, 0, pr.q, pr.N).tolist()]
    o0, o1 = R.keyswitch(pr, d, evk)
    got = R.phase(pr, o0, o1, s_eval, pr.L)
    want_eval = [[x * y % pr.q[i] for x, y in zip(d[i], s2_eval[i])] for i in range(pr.L)]
    want = R.poly_to_big(pr, want_eval, pr.L)
    Q = pr.Q(pr.L)
    err = max(abs(((g - w + Q // 2) % Q) - Q // 2) for g, w in zip(got, want))
    assert 0 < err <= _noise_bound(pr, pr.L)


# ------------------------------------------------------------------ hoisted rotation

def test_rotate_hoisted_identity_element_is_keyswitch_plus_c0():
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(3)
    s = ks_inputs.ternary_secret(1, pr.N)
    evk = _keys(pr, 5, s, s)
    c0 = _uniform_poly(rng, pr, range(pr.L))
    c1 = _uniform_poly(rng, pr, range(pr.L))
    (r0, r1), = R.rotate_hoisted(pr, (c0, c1), [1], [evk])
    k0, k1 = R.keyswitch(pr, c1, evk)
    assert r1 == k1
    assert r0 == [[(x + y) % pr.q[i] for x, y in zip(k0[i], c0[i])] for i in range(pr.L)]


@pytest.mark.parametrize("g", [5, 25, 61])
def test_rotate_hoisted_decrypts_to_rotated_phase(g):
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(g)
    s = ks_inputs.ternary_secret(1, pr.N)
    rot_key = _keys(pr, 9, R.automorphism_signed(s, g), s)
    ids = list(range(pr.L))
    s_eval = R.to_eval(pr, s, ids)
    # an honest ciphertext of a small message so that the phase is well inside Q
    msg = [rng.randrange(-1000, 1000) for _ in range(pr.N)]
    c1 = _uniform_poly(rng, pr, ids)
    mu = R.to_eval(pr, msg, ids)
    c0 = [[(mm - a * sv) % pr.q[i] for mm, a, sv in zip(mu[i], c1[i], s_eval[i])] for i in ids]
    (r0, r1), = R.rotate_hoisted(pr, (c0, c1), [g], [rot_key])
    got = R.phase(pr, r0, r1, s_eval, pr.L)
    want = R.automorphism_signed(msg, g)
    assert max(abs(a - b) for a, b in zip(got, want)) <= _noise_bound(pr, pr.L)


# ------------------------------------------------------------------ multiply, relinearise, rescale

def test_rotate_mac_with_unit_plaintext_is_rotate_hoisted():
    """Double-hoisted form, special case fixed by the single-hoisted one: one rotation, pt = 1."""
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(31)
    ids, all_ids = list(range(pr.L)), list(range(pr.L + pr.K))
    ct = (_uniform_poly(rng, pr, ids), _uniform_poly(rng, pr, ids))
    key = [[_uniform_poly(rng, pr, all_ids) for _ in range(2)] for _ in range(len(pr.digits(pr.L)))]
    one = [[1] * pr.N for _ in all_ids]
    for g in (5, 25):
        assert R.rotate_mac_hoisted(pr, ct, [g], [key], [one]) == R.rotate_hoisted(pr, ct, [g], [key])[0]
    zero = [[0] * pr.N for _ in all_ids]
    z0, z1 = R.rotate_mac_hoisted(pr, ct, [5], [key], [zero])
    assert all(v == 0 for limb in z0 + z1 for v in limb)


@pytest.mark.parametrize("ell", [4, 3])
def test_rotate_mac_decrypts_to_sum_of_plaintext_times_rotations(ell):
    """phase(out) = sum_r pt_r * sigma_{g_r}(phase(ct)) up to the key-switch noise of each rotation times its
    plaintext's 1-norm, plus one ModDown rounding."""
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(32)
    ids, all_ids = list(range(ell)), list(range(pr.L + pr.K))
    s = ks_inputs.ternary_secret(3, pr.N)
    s_eval = R.to_eval(pr, s, all_ids)
    galois = [5, 25, 125 % (2 * pr.N)]
    keys = [_keys(pr, 50 + r, R.automorphism_signed(s, g), s) for r, g in enumerate(galois)]
    pts_signed = [[rng.choice([-2, -1, 0, 0, 0, 1, 3]) for _ in range(pr.N)] for _ in galois]
    pts = [R.to_eval(pr, w, all_ids) for w in pts_signed]
    msg = [rng.randrange(-10**12, 10**12) for _ in range(pr.N)]   # every term of the sum dwarfs the noise bound
    a = _uniform_poly(rng, pr, ids)
    mu = R.to_eval(pr, msg, ids)
    b = [[(mm - x * sv) % pr.q[i] for mm, x, sv in zip(mu[i], a[i], s_eval[i])] for i in ids]
    o0, o1 = R.rotate_mac_hoisted(pr, (b, a), galois, keys, pts, ell)
    got = R.phase(pr, o0, o1, s_eval[:ell], ell)
    want = [0] * pr.N
    for g, w in zip(galois, pts_signed):
        term = R.poly_mul_signed(w, R.automorphism_signed(msg, g))
        want = [x + y for x, y in zip(want, term)]
    l1 = sum(sum(abs(x) for x in w) for w in pts_signed)
    # before the division, phase(u) = P sum_r pt_r sigma_r(phase) + sum_r pt_r sum_j sigma_r(d~_j) e_{r,j} with d~_j < alpha_j D_j < alpha_j P
    bound = l1 * pr.N * 19 * pr.L + pr.K * (pr.N + 1)
    assert max(abs(x - y) for x, y in zip(got, want)) <= bound


def test_bsgs_special_cases_reduce_to_the_single_level_operations():
    """One identity giant step: the outer level adds P v and divides by P again, exactly v.  One identity baby step with
    pt = 1 and one giant step G: a plain hoisted rotation by G."""
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(33)
    ids, all_ids = list(range(pr.L)), list(range(pr.L + pr.K))
    ct = (_uniform_poly(rng, pr, ids), _uniform_poly(rng, pr, ids))
    mk = lambda: [[_uniform_poly(rng, pr, all_ids) for _ in range(2)] for _ in range(len(pr.digits(pr.L)))]
    keys = [None, mk(), mk()]
    galois = [1, 5, 25]
    pts = [_uniform_poly(rng, pr, all_ids) for _ in galois]
    assert R.bsgs_linear_transform(pr, ct, galois, keys, [1], [None], [pts]) == R.rotate_mac_hoisted(pr, ct, galois, keys, pts)
    gk = mk()
    assert R.bsgs_linear_transform(pr, ct, [1], [None], [125 % (2 * pr.N)], [gk], [[None]]) == \
        R.rotate_hoisted(pr, ct, [125 % (2 * pr.N)], [gk])[0]


def test_bsgs_decrypts_to_the_double_sum():
    """phase(out) = sum_g sigma_{G_g}( sum_b pt_{g,b} sigma_{B_b}(message) ) up to key-switch noise."""
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(34)
    ell = pr.L
    ids, all_ids = list(range(ell)), list(range(pr.L + pr.K))
    s = ks_inputs.ternary_secret(4, pr.N)
    s_eval = R.to_eval(pr, s, all_ids)
    baby, giant = [1, 5, 25], [1, 125 % (2 * pr.N)]
    key_for = lambda seed, g: None if g == 1 else _keys(pr, seed, R.automorphism_signed(s, g), s)
    bkeys = [key_for(60 + i, g) for i, g in enumerate(baby)]
    gkeys = [key_for(70 + i, g) for i, g in enumerate(giant)]
    w_signed = [[[rng.choice([-2, -1, 0, 0, 1, 2]) for _ in range(pr.N)] for _ in baby] for _ in giant]
    pts = [[R.to_eval(pr, w, all_ids) for w in row] for row in w_signed]
    msg = [rng.randrange(-10**12, 10**12) for _ in range(pr.N)]
    a = _uniform_poly(rng, pr, ids)
    mu = R.to_eval(pr, msg, ids)
    b = [[(mm - x * sv) % pr.q[i] for mm, x, sv in zip(mu[i], a[i], s_eval[i])] for i in ids]
    o0, o1 = R.bsgs_linear_transform(pr, (b, a), baby, bkeys, giant, gkeys, pts, ell)
    got = R.phase(pr, o0, o1, s_eval[:ell], ell)
    want = [0] * pr.N
    for G, row in zip(giant, w_signed):
        inner = [0] * pr.N
        for Bb, w in zip(baby, row):
            inner = [x + y for x, y in zip(inner, R.poly_mul_signed(w, R.automorphism_signed(msg, Bb)))]
        want = [x + y for x, y in zip(want, R.automorphism_signed(inner, G))]
    l1 = max(sum(sum(abs(x) for x in w) for w in row) for row in w_signed)
    ks_noise = pr.N * 19 * pr.L + pr.K * (pr.N + 1)
    bound = len(giant) * (l1 * ks_noise + ks_noise)      # inner sums' noise passes through the outer rotations, which add their own
    assert max(abs(x - y) for x, y in zip(got, want)) <= bound


def test_rescale_is_rounded_division():
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(11)
    ell = 4
    c = _uniform_poly(rng, pr, range(ell))
    out = R.rescale(pr, c, ell)
    big = R.poly_to_big(pr, c, ell)
    ql = pr.q[ell - 1]
    got = R.poly_to_big(pr, out, ell - 1)
    Qn = pr.Q(ell - 1)
    for v, g in zip(big, got):
        rounded = (2 * v + ql) // (2 * ql)          # round to nearest; q odd, so no ties
        assert (g - rounded) % Qn == 0


def test_hmult_relin_rescale_phase_identity():
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(12)
    ids = list(range(pr.L))
    all_ids = list(range(pr.L + pr.K))
    s = ks_inputs.ternary_secret(1, pr.N)
    s_eval_all = R.to_eval(pr, s, all_ids)
    s2_signed = R.poly_mul_signed(s, s)
    rlk = _keys(pr, 21, s2_signed, s)
    s_eval = s_eval_all[:pr.L]

    def encrypt(msg):
        a = _uniform_poly(rng, pr, ids)
        mu = R.to_eval(pr, msg, ids)
        b = [[(mm - x * sv) % pr.q[i] for mm, x, sv in zip(mu[i], a[i], s_eval[i])] for i in ids]
        return b, a

    scale = pr.q[pr.L - 1]
    m1 = [rng.randrange(-50, 50) * scale // 64 for _ in range(pr.N)]
    m2 = [rng.randrange(-50, 50) * scale // 64 for _ in range(pr.N)]
    cta, ctb = encrypt(m1), encrypt(m2)
    o0, o1 = R.hmult_relin_rescale(pr, cta, ctb, rlk)
    got = R.phase(pr, o0, o1, s_eval[:pr.L - 1], pr.L - 1)
    prod = R.poly_mul_signed(m1, m2)
    # phase' * q_last = phase +- q_last (N + 1) / 2, and phase = m1 m2 + key-switch noise
    bound = (_noise_bound(pr, pr.L) // scale) + (pr.N + 1) // 2 + 2
    assert max(abs(g - (2 * w + scale) // (2 * scale)) for g, w in zip(got, prod)) <= bound


@pytest.mark.parametrize("L,K,dnum,ell", [(4, 2, 2, 4), (5, 3, 2, 4), (3, 1, 3, 3)])
def test_mod_down_merged_is_floor_division_by_P_qlast(L, K, dnum, ell):
    """Pin for the merged ModDown + rescale: with X = acc + P * addend as an integer modulo P Q_ell (CRT of the
    inputs, independent of the oracle's own arithmetic), every output coefficient is floor(X / (P q_last)) - u with
    0 <= u <= K (the lift error of a fast conversion from K + 1 sources)."""
    pr = _small_params(4, L, K, dnum)
    rng = random.Random(40 + L)
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    acc = _uniform_poly(rng, pr, ext_ids)
    addend = _uniform_poly(rng, pr, range(ell))
    out = R.mod_down_merged(pr, acc, addend, ell)
    ext_mods = [pr.moduli[m] for m in ext_ids]
    acc_coeff = [R.intt(acc[pos], pr.moduli[m], pr.psi[m]) for pos, m in enumerate(ext_ids)]
    add_coeff = [R.intt(addend[i], pr.q[i], pr.psi[i]) for i in range(ell)]
    out_coeff = [R.intt(out[i], pr.q[i], pr.psi[i]) for i in range(ell - 1)]
    PQ = pr.P * pr.Q(ell)
    D = pr.P * pr.q[ell - 1]
    Qn = pr.Q(ell - 1)
    seen_u = set()
    for n in range(pr.N):
        X = (R.crt_reconstruct([limb[n] for limb in acc_coeff], ext_mods)
             + pr.P * R.crt_reconstruct([limb[n] for limb in add_coeff], pr.q[:ell])) % PQ
        got = R.crt_reconstruct([limb[n] for limb in out_coeff], pr.q[:ell - 1])
        u = (X // D - got) % Qn
        assert 0 <= u <= pr.K, (n, u)
        seen_u.add(u)
    assert len(seen_u) > 1 or pr.K == 0     # the lift error really occurs: the test would notice a centred variant


@pytest.mark.parametrize("L,K,dnum,ell", [(4, 2, 2, 4), (5, 3, 2, 4), (3, 1, 3, 3)])
def test_mod_down_is_floor_division_by_P_with_lift_error(L, K, dnum, ell):
    """Pin that tells the fast conversion from the exact one inside mod_down: with X the CRT reconstruction of the
    accumulator modulo P Q_ell (computed here, not by the function under test), every output coefficient is
    floor(X / P) - v with 0 <= v < K, and v > 0 really occurs -- an exact (corrected) conversion would give v = 0
    everywhere, a centred one negative v."""
    pr = _small_params(4, L, K, dnum)
    rng = random.Random(50 + L)
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    ext_mods = [pr.moduli[m] for m in ext_ids]
    acc = _uniform_poly(rng, pr, ext_ids)
    out = R.mod_down(pr, acc, ell)
    acc_coeff = [R.intt(acc[pos], pr.moduli[m], pr.psi[m]) for pos, m in enumerate(ext_ids)]
    out_coeff = [R.intt(out[i], pr.q[i], pr.psi[i]) for i in range(ell)]
    Q = pr.Q(ell)
    seen = set()
    for n in range(pr.N):
        X = R.crt_reconstruct([limb[n] for limb in acc_coeff], ext_mods)
        got = R.crt_reconstruct([limb[n] for limb in out_coeff], pr.q[:ell])
        v = (X // pr.P - got) % Q
        assert 0 <= v < max(pr.K, 1), (n, v)
        seen.add(v)
    assert pr.K == 1 or len(seen) > 1


@pytest.mark.parametrize("L,K,dnum,ell", [(4, 2, 2, 4), (5, 3, 2, 5), (6, 2, 2, 5)])
def test_mod_up_limbs_are_the_digit_value_plus_lift_error(L, K, dnum, ell):
    """The same for mod_up: the raised limbs of digit j are congruent to x + u D_j, x the digit's value in [0, D_j)
    (CRT of its limbs, computed here) and 0 <= u < alpha_j the same for every target modulus of a coefficient;
    u > 0 occurs, which an exact conversion would never produce."""
    pr = _small_params(4, L, K, dnum)
    rng = random.Random(60 + L)
    d = _uniform_poly(rng, pr, range(ell))
    lifted = R.mod_up(pr, d, ell)
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    d_coeff = [R.intt(d[i], pr.q[i], pr.psi[i]) for i in range(ell)]
    for j, dig in enumerate(pr.digits(ell)):
        src = [pr.q[i] for i in dig]
        Dj = 1
        for q in src:
            Dj *= q
        lifted_coeff = [R.intt(lifted[j][pos], pr.moduli[m], pr.psi[m]) for pos, m in enumerate(ext_ids)]
        seen = set()
        for n in range(pr.N):
            x = R.crt_reconstruct([d_coeff[i][n] for i in dig], src)
            us = set()
            for pos, m in enumerate(ext_ids):
                t = pr.moduli[m]
                if m in dig:
                    assert lifted_coeff[pos][n] == x % t
                    continue
                # u from this target: (limb - x) / D_j modulo t
                us.add((lifted_coeff[pos][n] - x) * pow(Dj % t, -1, t) % t)
            assert len(us) == 1, (j, n, us)          # one lift error per coefficient, shared by all targets
            u = us.pop()
            assert 0 <= u < len(dig), (j, n, u)
            seen.add(u)
        assert len(dig) == 1 or len(seen) > 1


def test_hmult_merged_decrypts_to_scaled_product():
    pr = _small_params(5, 4, 2, 2)
    rng = random.Random(12)
    ids = list(range(pr.L))
    all_ids = list(range(pr.L + pr.K))
    s = ks_inputs.ternary_secret(1, pr.N)
    s_eval = R.to_eval(pr, s, all_ids)[:pr.L]
    rlk = _keys(pr, 21, R.poly_mul_signed(s, s), s)

    def encrypt(msg):
        a = _uniform_poly(rng, pr, ids)
        mu = R.to_eval(pr, msg, ids)
        return [[(mm - x * sv) % pr.q[i] for mm, x, sv in zip(mu[i], a[i], s_eval[i])] for i in ids], a

    scale = pr.q[pr.L - 1]
    m1 = [rng.randrange(-50, 50) * scale // 64 for _ in range(pr.N)]
    m2 = [rng.randrange(-50, 50) * scale // 64 for _ in range(pr.N)]
    cta, ctb = encrypt(m1), encrypt(m2)
    o0, o1 = R.hmult_relin_rescale_merged(pr, cta, ctb, rlk)
    got = R.phase(pr, o0, o1, s_eval[:pr.L - 1], pr.L - 1)
    prod = R.poly_mul_signed(m1, m2)
    # each component is floor(.) - u, u <= K: the phase is off by at most (K + 1)(1 + |s|_1) from phase / q_last
    bound = (_noise_bound(pr, pr.L) // scale) + (pr.K + 2) * (pr.N + 1) + 2
    assert max(abs(g - w // scale) for g, w in zip(got, prod)) <= bound
    # and it agrees with the unmerged chain up to the two roundings
    u0, u1 = R.hmult_relin_rescale(pr, cta, ctb, rlk)
    ref = R.phase(pr, u0, u1, s_eval[:pr.L - 1], pr.L - 1)
    assert max(abs(g - r) for g, r in zip(got, ref)) <= (pr.K + 3) * (pr.N + 1)
    assert (o0, o1) != (u0, u1)


def test_tensor_product_matches_polynomial_identity():
    pr = _small_params(4, 3, 1, 1)
    rng = random.Random(13)
    ids = list(range(pr.L))
    cta = (_uniform_poly(rng, pr, ids), _uniform_poly(rng, pr, ids))
    ctb = (_uniform_poly(rng, pr, ids), _uniform_poly(rng, pr, ids))
    d0, d1, d2 = R.tensor_product(pr, cta, ctb, pr.L)
    # (b1 + a1 Y)(b2 + a2 Y) = d0 + d1 Y + d2 Y^2 at a random point Y, slot-wise
    for i in ids:
        qi = pr.q[i]
        Y = rng.randrange(qi)
        for n in range(pr.N):
            lhs = (cta[0][i][n] + cta[1][i][n] * Y) * (ctb[0][i][n] + ctb[1][i][n] * Y) % qi
            assert lhs == (d0[i][n] + d1[i][n] * Y + d2[i][n] * Y * Y) % qi
