"""Reference tier (i): CKKS hybrid key-switching over RNS polynomials in plain Python integers.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
GPU library must compute.  It shares no code with the HIP path and nothing in the product
package may import it; only tests, the smoke check and the benchmark's cpu_baseline leg do.

The paper names the operations (Background: "RNS and Limbs", "NTT", "Evaluation Keys";
Motivation: hoisting; Kernel Code Generation: the NTT / Base Conversion / Elementwise kernel
classes) but prints no formula for any of them, so every function below follows the textbook
definition from the work the paper cites for that operation (hybrid key-switching with special
primes, fast RNS base conversion, hoisted rotations) under the readings listed in the design
notes.  Every function is pinned by tests against something other than itself: brute-force
negacyclic convolution, big-integer CRT reconstruction, closed forms with a transparent key and
the decrypt-within-noise bound.  Parity unpinned: none.

Conventions
-----------
* A polynomial over one modulus is a Python list of N ints in [0, m).
* A multi-limb polynomial is a list of such lists, one per modulus, N contiguous.
* Evaluation ("NTT") domain order is bit-reversed: slot k holds a(psi^(2*brv(k)+1)).
* Moduli are indexed 0..L+K-1: ciphertext primes q_0..q_{L-1} then special primes p_0..p_{K-1}.
"""

from __future__ import annotations


# --------------------------------------------------------------------------------------
# parameters: primes, roots of unity, bit reversal
# --------------------------------------------------------------------------------------

def is_prime(n: int) -> bool:
    """Deterministic Miller-Rabin for n < 3.3e24 (first 13 primes as witnesses)."""
    if n < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41)
    for p in small:
        if n % p == 0:
            return n == p
    d, s = n - 1, 0
    while d % 2 == 0:
        d //= 2
        s += 1
    for a in small:
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


def ntt_primes(logN: int, count: int, bits: int = 36) -> list[int]:
    """The `count` largest primes below 2^bits with m = 1 (mod 2N), in descending order.

    Workload recipe: special primes are the first K of this list, ciphertext primes the next L
    (so P exceeds every digit product)."""
    step = 2 << logN
    m = (1 << bits) + 1 - step
    out = []
    while len(out) < count:
        if m <= step:
            raise ValueError("ran out of candidates")
        if is_prime(m):
            out.append(m)
        m -= step
    return out


def minimal_psi(m: int, logN: int) -> int:
    """Smallest positive integer psi with psi^N = -1 (mod m): a primitive 2N-th root of unity.

    All N such roots are the odd powers of any one of them, so enumerate those and take the least."""
    N = 1 << logN
    x = 2
    while True:
        root = pow(x, (m - 1) // (2 * N), m)
        if pow(root, N, m) == m - 1:
            break
        x += 1
    sq = root * root % m
    best, cur = root, root
    for _ in range(N - 1):
        cur = cur * sq % m
        if cur < best:
            best = cur
    return best


def brv(k: int, bits: int) -> int:
    r = 0
    for _ in range(bits):
        r = (r << 1) | (k & 1)
        k >>= 1
    return r


# --------------------------------------------------------------------------------------
# negacyclic ring arithmetic and the transform (Background, "NTT")
# --------------------------------------------------------------------------------------

def negacyclic_mul(a: list[int], b: list[int], m: int) -> list[int]:
    """Schoolbook product in Z_m[X]/(X^N + 1): X^N wraps around with a sign flip."""
    N = len(a)
    c = [0] * N
    for i, ai in enumerate(a):
        if ai == 0:
            continue
        for j, bj in enumerate(b):
            k = i + j
            if k < N:
                c[k] = (c[k] + ai * bj) % m
            else:
                c[k - N] = (c[k - N] - ai * bj) % m
    return c


def ntt_def(a: list[int], m: int, psi: int) -> list[int]:
    """The transform by its definition: out[k] = a(psi^(2*brv(k)+1)) = sum_i a_i psi^((2 brv(k)+1) i)."""
    N = len(a)
    logN = N.bit_length() - 1
    out = []
    for k in range(N):
        x = pow(psi, 2 * brv(k, logN) + 1, m)
        acc, xp = 0, 1
        for ai in a:
            acc = (acc + ai * xp) % m
            xp = xp * x % m
        out.append(acc)
    return out


def intt_def(A: list[int], m: int, psi: int) -> list[int]:
    """Inverse of ntt_def by its definition: a_i = N^-1 sum_k A[k] psi^(-(2 brv(k)+1) i)."""
    N = len(A)
    logN = N.bit_length() - 1
    ninv = pow(N, -1, m)
    psiinv = pow(psi, -1, m)
    xs = [pow(psiinv, 2 * brv(k, logN) + 1, m) for k in range(N)]
    out = []
    for i in range(N):
        acc = 0
        for k in range(N):
            acc = (acc + A[k] * pow(xs[k], i, m)) % m
        out.append(acc * ninv % m)
    return out


def ntt(a: list[int], m: int, psi: int) -> list[int]:
    """Textbook iterative decimation-in-time transform, natural order in, bit-reversed order out.

    Stage with `half` = distance between butterfly partners; block b of that stage multiplies its
    lower half by psi^brv(blocks + b) where blocks = N/(2*half)."""
    N = len(a)
    logN = N.bit_length() - 1
    a = list(a)
    blocks, half = 1, N // 2
    while half >= 1:
        for b in range(blocks):
            w = pow(psi, brv(blocks + b, logN), m)
            lo = 2 * b * half
            for j in range(lo, lo + half):
                t = a[j + half] * w % m
                a[j + half] = (a[j] - t) % m
                a[j] = (a[j] + t) % m
        blocks, half = blocks * 2, half // 2
    return a


def intt(A: list[int], m: int, psi: int) -> list[int]:
    """Undo `ntt` stage by stage (decimation-in-frequency), then scale by N^-1."""
    N = len(A)
    logN = N.bit_length() - 1
    a = list(A)
    psiinv = pow(psi, -1, m)
    blocks, half = N // 2, 1
    while blocks >= 1:
        for b in range(blocks):
            w = pow(psiinv, brv(blocks + b, logN), m)
            lo = 2 * b * half
            for j in range(lo, lo + half):
                u, v = a[j], a[j + half]
                a[j] = (u + v) % m
                a[j + half] = (u - v) * w % m
        blocks, half = blocks // 2, half * 2
    ninv = pow(N, -1, m)
    return [x * ninv % m for x in a]


def automorphism_coeff(a: list[int], g: int, m: int) -> list[int]:
    """sigma_g: a(X) -> a(X^g) in Z_m[X]/(X^N+1), g odd.  X^i goes to +-X^(i g mod N)."""
    N = len(a)
    out = [0] * N
    for i, ai in enumerate(a):
        e = i * g % (2 * N)
        if e < N:
            out[e] = ai
        else:
            out[e - N] = (m - ai) % m
    return out


def automorphism_eval(A: list[int], g: int) -> list[int]:
    """sigma_g on a bit-reversed evaluation vector: a pure permutation.

    (sigma_g a)(x) = a(x^g); slot k holds x = psi^(2 brv(k)+1), so it takes the slot holding
    psi^(g (2 brv(k)+1) mod 2N)."""
    N = len(A)
    logN = N.bit_length() - 1
    out = [0] * N
    for k in range(N):
        e = g * (2 * brv(k, logN) + 1) % (2 * N)
        out[k] = A[brv((e - 1) // 2, logN)]
    return out


# --------------------------------------------------------------------------------------
# RNS base conversion (Kernel Code Generation: "Base Conversion" kernel class)
# --------------------------------------------------------------------------------------

def bconv_lift(x: list[int], src: list[int]) -> int:
    """The integer the fast conversion implicitly lifts one coefficient to:
    X~ = sum_i [x_i (D/q_i)^-1]_{q_i} * (D/q_i), an exact integer with X~ = x + u D, 0 <= u < len(src)."""
    D = 1
    for q in src:
        D *= q
    total = 0
    for xi, q in zip(x, src):
        Dhat = D // q
        y = xi * pow(Dhat % q, -1, q) % q
        total += y * Dhat
    return total


def bconv_fast(x_limbs: list[list[int]], src: list[int], dst: list[int]) -> list[list[int]]:
    """Fast (uncorrected) base conversion, coefficient-wise: out_t = X~ mod t for every t in dst."""
    N = len(x_limbs[0])
    out = [[0] * N for _ in dst]
    for n in range(N):
        lifted = bconv_lift([limb[n] for limb in x_limbs], src)
        for ti, t in enumerate(dst):
            out[ti][n] = lifted % t
    return out


def crt_reconstruct(x: list[int], src: list[int]) -> int:
    """The unique integer in [0, D) with the given residues."""
    D = 1
    for q in src:
        D *= q
    return bconv_lift(x, src) % D


def bconv_exact(x_limbs: list[list[int]], src: list[int], dst: list[int]) -> list[list[int]]:
    """Exact conversion of the representative in [0, D): used for invariants only."""
    N = len(x_limbs[0])
    out = [[0] * N for _ in dst]
    for n in range(N):
        v = crt_reconstruct([limb[n] for limb in x_limbs], src)
        for ti, t in enumerate(dst):
            out[ti][n] = v % t
    return out


# --------------------------------------------------------------------------------------
# parameter bundle
# --------------------------------------------------------------------------------------

class Params:
    """Ring degree, RNS basis q_0..q_{L-1} | p_0..p_{K-1}, digit partition for hybrid key-switching."""

    def __init__(self, logN: int, q: list[int], p: list[int], dnum: int, psi: list[int] | None = None):
        self.logN, self.N = logN, 1 << logN
        self.q, self.p = list(q), list(p)
        self.L, self.K, self.dnum = len(q), len(p), dnum
        self.moduli = self.q + self.p
        self.psi = list(psi) if psi is not None else [minimal_psi(m, logN) for m in self.moduli]
        self.alpha = -(-self.L // dnum)
        self.P = 1
        for pk in self.p:
            self.P *= pk

    def digits(self, ell: int) -> list[list[int]]:
        """Contiguous digits of alpha limbs covering limbs 0..ell-1; the last may be short."""
        return [list(range(s, min(s + self.alpha, ell))) for s in range(0, ell, self.alpha)]

    def Q(self, ell: int) -> int:
        Q = 1
        for qi in self.q[:ell]:
            Q *= qi
        return Q


# --------------------------------------------------------------------------------------
# hybrid key-switching (Background, "Evaluation Keys"; the chain INTT, ModUp, NTT, inner
# product, INTT, ModDown, NTT)
# --------------------------------------------------------------------------------------

def mod_up(pr: Params, d_eval: list[list[int]], ell: int) -> list[list[list[int]]]:
    """Decompose and raise: for every digit j return d~_j on all ell+K moduli in evaluation domain.

    Limbs inside the digit are the input limbs unchanged; every other limb is the fast base
    conversion of the digit's coefficient-domain limbs, transformed to evaluation domain.
    Index order of the returned limbs: q_0..q_{ell-1}, p_0..p_{K-1}."""
    coeff = [intt(d_eval[i], pr.q[i], pr.psi[i]) for i in range(ell)]
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    lifted = []
    for dig in pr.digits(ell):
        src = [pr.q[i] for i in dig]
        dst_ids = [m for m in ext_ids if m not in dig]
        conv = bconv_fast([coeff[i] for i in dig], src, [pr.moduli[m] for m in dst_ids])
        limbs = []
        for m in ext_ids:
            if m in dig:
                limbs.append(list(d_eval[m]))
            else:
                c = conv[dst_ids.index(m)]
                limbs.append(ntt(c, pr.moduli[m], pr.psi[m]))
        lifted.append(limbs)
    return lifted


def inner_product(pr: Params, lifted, evk, ell: int):
    """acc_c[m] = sum_j d~_j[m] * evk[j][c][m]  (slot-wise, mod the limb's modulus).

    evk[j][c] carries all L+K limbs; at level ell only limbs q_0..q_{ell-1} and p_* are used."""
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    acc = [[[0] * pr.N for _ in ext_ids] for _ in range(2)]
    for j, dj in enumerate(lifted):
        for c in range(2):
            for pos, m in enumerate(ext_ids):
                mod = pr.moduli[m]
                key = evk[j][c][m]
                row = acc[c][pos]
                src = dj[pos]
                for n in range(pr.N):
                    row[n] = (row[n] + src[n] * key[n]) % mod
    return acc


def mod_down(pr: Params, acc_c: list[list[int]], ell: int) -> list[list[int]]:
    """Divide by P: out[i] = (acc[i] - NTT(BConv_{P -> q_i}(INTT(acc on p-limbs)))) * P^-1 mod q_i."""
    special = [intt(acc_c[ell + k], pr.p[k], pr.psi[pr.L + k]) for k in range(pr.K)]
    conv = bconv_fast(special, pr.p, pr.q[:ell])
    out = []
    for i in range(ell):
        qi = pr.q[i]
        w = ntt(conv[i], qi, pr.psi[i])
        pinv = pow(pr.P % qi, -1, qi)
        out.append([(a - b) * pinv % qi for a, b in zip(acc_c[i], w)])
    return out


def keyswitch(pr: Params, d_eval: list[list[int]], evk, ell: int | None = None):
    """Key-switch one polynomial d (ell limbs, evaluation domain): returns (out_0, out_1)."""
    ell = pr.L if ell is None else ell
    lifted = mod_up(pr, d_eval, ell)
    acc = inner_product(pr, lifted, evk, ell)
    return mod_down(pr, acc[0], ell), mod_down(pr, acc[1], ell)


def rotate_hoisted(pr: Params, ct, galois: list[int], rot_keys, ell: int | None = None):
    """Hoisted rotations of one ciphertext ct = (c0, c1): one decompose-and-raise of c1 is shared by
    all Galois elements (Motivation: hoisting).  For each g: apply sigma_g to the raised digits,
    inner product with that rotation's key, divide by P, add sigma_g(c0) to component 0.

    sigma_g is applied here in the coefficient domain, by its definition, around this file's own
    transform pair."""
    ell = pr.L if ell is None else ell
    c0, c1 = ct
    lifted = mod_up(pr, c1, ell)
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]

    def sigma_eval(limb, m, g):
        mod, psi = pr.moduli[m], pr.psi[m]
        return ntt(automorphism_coeff(intt(limb, mod, psi), g, mod), mod, psi)

    outs = []
    for g, key in zip(galois, rot_keys):
        rotated = [[sigma_eval(dj[pos], m, g) for pos, m in enumerate(ext_ids)] for dj in lifted]
        acc = inner_product(pr, rotated, key, ell)
        o0, o1 = mod_down(pr, acc[0], ell), mod_down(pr, acc[1], ell)
        for i in range(ell):
            s = sigma_eval(c0[i], i, g)
            o0[i] = [(a + b) % pr.q[i] for a, b in zip(o0[i], s)]
        outs.append((o0, o1))
    return outs


def _rotation_term(pr: Params, ct, lifted, g: int, key, ell: int):
    """One rotated ciphertext on the extended basis, before any division by P: the pair
    (acc_0 + P sigma_g(c0), acc_1) where acc is the inner product of the sigma_g-permuted raised digits
    of c1 with the rotation key.  g = 1 stands for the unrotated ciphertext: no key is involved and
    the pair is P (c0, c1).  (P x is x [P]_{q_i} on the ciphertext limbs and 0 on the special limbs.)"""
    c0, c1 = ct
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]

    def sigma_eval(limb, m):
        mod, psi = pr.moduli[m], pr.psi[m]
        return ntt(automorphism_coeff(intt(limb, mod, psi), g, mod), mod, psi)

    if g == 1:
        t = [[[0] * pr.N for _ in ext_ids] for _ in range(2)]
        for i in range(ell):
            pm = pr.P % pr.q[i]
            t[0][i] = [pm * x % pr.q[i] for x in c0[i]]
            t[1][i] = [pm * x % pr.q[i] for x in c1[i]]
        return t
    rotated = [[sigma_eval(dj[pos], m) for pos, m in enumerate(ext_ids)] for dj in lifted]
    acc = inner_product(pr, rotated, key, ell)
    for i in range(ell):
        pm = pr.P % pr.q[i]
        acc[0][i] = [(a + pm * b) % pr.q[i] for a, b in zip(acc[0][i], sigma_eval(c0[i], i))]
    return acc


def rotate_mac_hoisted(pr: Params, ct, galois: list[int], rot_keys, pts, ell: int | None = None):
    """Inner sum of a baby-step giant-step linear transform with the rotations kept in the extended
    basis ("double hoisting", the form in which the DSL's BSGS matrix products consume hoisted
    rotations): sum_r pt_r * rot_{g_r}(ct) with ONE division by P for the whole sum instead of one per
    rotation.

    For every Galois element g_r: the raised digits of c1 (one decompose-and-raise, shared) are
    permuted by sigma_{g_r} and multiplied with that rotation's key, which gives both accumulators on
    the extended basis; sigma_{g_r}(c0) joins component 0 lifted to that basis as P * sigma(c0)
    (_rotation_term; g_r = 1 is the unrotated ciphertext, P (c0, c1), and reads no key).  Each
    rotation's pair is multiplied slot-wise by the plaintext pt_r (evaluation domain, all L + K limbs,
    like a key; None = the constant 1) and the products are summed; the sum is divided by P once:

        u_c[m]  = sum_r pt_r[m] * term_{r,c}[m]   mod m,        out_c = mod_down(u_c).

    With one rotation g != 1 and pt = 1 this is rotate_hoisted bit for bit."""
    ell = pr.L if ell is None else ell
    lifted = mod_up(pr, ct[1], ell)
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    u = [[[0] * pr.N for _ in ext_ids] for _ in range(2)]
    for g, key, pt in zip(galois, rot_keys, pts):
        term = _rotation_term(pr, ct, lifted, g, key, ell)
        for c in range(2):
            for pos, m in enumerate(ext_ids):
                mod = pr.moduli[m]
                w = pt[m] if pt is not None else [1] * pr.N
                u[c][pos] = [(x + wv * a) % mod for x, wv, a in zip(u[c][pos], w, term[c][pos])]
    return mod_down(pr, u[0], ell), mod_down(pr, u[1], ell)


def bsgs_linear_transform(pr: Params, ct, baby_galois, baby_keys, giant_galois, giant_keys, pts, ell: int | None = None):
    """Baby-step giant-step linear transform (DSL, matrix multiplication example), double-hoisted at
    both levels:

        out = sum_g rot_{G_g}( sum_b pts[g][b] * rot_{B_b}(ct) ).

    Inner sums: rotate_mac_hoisted with the baby-step elements B_b (one decompose-and-raise of c1 for
    all of them, one division by P per giant step) give v_g on the ciphertext basis.  Outer sum: every
    v_g is rotated by its giant-step element G_g on the extended basis (_rotation_term: its own
    decompose-and-raise, key G_g; G_g = 1 adds P v_g), the terms are added and divided by P once."""
    ell = pr.L if ell is None else ell
    ext_ids = list(range(ell)) + [pr.L + k for k in range(pr.K)]
    u = [[[0] * pr.N for _ in ext_ids] for _ in range(2)]
    for G, gkey, row in zip(giant_galois, giant_keys, pts):
        v = rotate_mac_hoisted(pr, ct, baby_galois, baby_keys, row, ell)
        term = _rotation_term(pr, v, mod_up(pr, v[1], ell) if G != 1 else None, G, gkey, ell)
        for c in range(2):
            for pos, m in enumerate(ext_ids):
                mod = pr.moduli[m]
                u[c][pos] = [(x + a) % mod for x, a in zip(u[c][pos], term[c][pos])]
    return mod_down(pr, u[0], ell), mod_down(pr, u[1], ell)


def tensor_product(pr: Params, cta, ctb, ell: int):
    """(b1,a1) x (b2,a2) -> d0 = b1 b2, d1 = a1 b2 + a2 b1, d2 = a1 a2, slot-wise per limb."""
    (b1, a1), (b2, a2) = cta, ctb
    d0, d1, d2 = [], [], []
    for i in range(ell):
        qi = pr.q[i]
        d0.append([x * y % qi for x, y in zip(b1[i], b2[i])])
        d1.append([(x * y + z * w) % qi for x, y, z, w in zip(a1[i], b2[i], a2[i], b1[i])])
        d2.append([x * y % qi for x, y in zip(a1[i], a2[i])])
    return d0, d1, d2


def rescale(pr: Params, c: list[list[int]], ell: int) -> list[list[int]]:
    """Drop the last limb q_{ell-1} with rounding to nearest: subtract the centred remainder
    modulo q_{ell-1}, then divide exactly by q_{ell-1}, limb by limb."""
    ql = pr.q[ell - 1]
    r = intt(c[ell - 1], ql, pr.psi[ell - 1])
    half = (ql - 1) // 2
    out = []
    for i in range(ell - 1):
        qi = pr.q[i]
        rc = [(x - ql) % qi if x > half else x % qi for x in r]
        w = ntt(rc, qi, pr.psi[i])
        qlinv = pow(ql % qi, -1, qi)
        out.append([(a - b) * qlinv % qi for a, b in zip(c[i], w)])
    return out


def hmult_relin_rescale(pr: Params, cta, ctb, rlk, ell: int | None = None):
    """Homomorphic multiply: tensor product, key-switch d2 with the relinearisation key, add,
    rescale both components.  Returns (out_0, out_1) on ell-1 limbs."""
    ell = pr.L if ell is None else ell
    d0, d1, d2 = tensor_product(pr, cta, ctb, ell)
    k0, k1 = keyswitch(pr, d2, rlk, ell)
    c0 = [[(x + y) % pr.q[i] for x, y in zip(d0[i], k0[i])] for i in range(ell)]
    c1 = [[(x + y) % pr.q[i] for x, y in zip(d1[i], k1[i])] for i in range(ell)]
    return rescale(pr, c0, ell), rescale(pr, c1, ell)


def mod_down_merged(pr: Params, acc_c: list[list[int]], addend: list[list[int]], ell: int) -> list[list[int]]:
    """ModDown merged with the rescale that follows it (Compiler, polynomial-level optimisations:
    "mod down merging"): instead of dividing by P and then by q_{ell-1}, add P * addend on the
    ciphertext limbs (the addend is what the division by P would have been added to: d0 or d1 of a
    multiplication) and divide once by D = P * q_{ell-1}, with one base conversion from the basis
    {p_0..p_{K-1}, q_{ell-1}} to q_0..q_{ell-2}:

        acc'[i]   = acc[i] + [P]_{q_i} * addend[i]            i < ell   (special limbs unchanged: P = 0 there)
        out[i]    = (acc'[i] - NTT(BConv_{S -> q_i}(INTT(acc' on S)))) * D^-1 mod q_i,   i < ell - 1.

    The fast conversion lifts [acc']_D to [acc']_D + u D with 0 <= u <= K, so every coefficient of
    the result is floor(acc' / D) - u: floor-type rounding throughout, where the unmerged chain
    floors the division by P and rounds the division by q_{ell-1} to nearest."""
    ql = pr.q[ell - 1]
    accp = [[(a + (pr.P % pr.q[i]) * d) % pr.q[i] for a, d in zip(acc_c[i], addend[i])] for i in range(ell)]
    src = list(pr.p) + [ql]
    src_limbs = [intt(acc_c[ell + k], pr.p[k], pr.psi[pr.L + k]) for k in range(pr.K)]
    src_limbs.append(intt(accp[ell - 1], ql, pr.psi[ell - 1]))
    conv = bconv_fast(src_limbs, src, pr.q[:ell - 1])
    D = pr.P * ql
    out = []
    for i in range(ell - 1):
        qi = pr.q[i]
        w = ntt(conv[i], qi, pr.psi[i])
        dinv = pow(D % qi, -1, qi)
        out.append([(a - b) * dinv % qi for a, b in zip(accp[i], w)])
    return out


def hmult_relin_rescale_merged(pr: Params, cta, ctb, rlk, ell: int | None = None):
    """Homomorphic multiply with the relinearisation's ModDown and the rescale merged into one
    division by P * q_{ell-1} (mod_down_merged).  Returns (out_0, out_1) on ell-1 limbs."""
    ell = pr.L if ell is None else ell
    d0, d1, d2 = tensor_product(pr, cta, ctb, ell)
    lifted = mod_up(pr, d2, ell)
    acc0, acc1 = inner_product(pr, lifted, rlk, ell)
    return mod_down_merged(pr, acc0, d0, ell), mod_down_merged(pr, acc1, d1, ell)


# --------------------------------------------------------------------------------------
# textbook key generation, encryption, decryption (host side only)
# --------------------------------------------------------------------------------------

def to_eval(pr: Params, poly_signed: list[int], mod_ids: list[int]) -> list[list[int]]:
    """Small signed integer polynomial -> evaluation-domain limbs on the given moduli."""
    return [ntt([x % pr.moduli[m] for x in poly_signed], pr.moduli[m], pr.psi[m]) for m in mod_ids]


def poly_mul_signed(a: list[int], b: list[int]) -> list[int]:
    """Negacyclic product over the integers (no modulus)."""
    N = len(a)
    c = [0] * N
    for i, ai in enumerate(a):
        if ai == 0:
            continue
        for j, bj in enumerate(b):
            k = i + j
            if k < N:
                c[k] += ai * bj
            else:
                c[k - N] -= ai * bj
    return c


def automorphism_signed(a: list[int], g: int) -> list[int]:
    N = len(a)
    out = [0] * N
    for i, ai in enumerate(a):
        e = i * g % (2 * N)
        if e < N:
            out[e] = ai
        else:
            out[e - N] = -ai
    return out


def switching_key(pr: Params, s_from_eval: list[list[int]], s_to_eval: list[list[int]],
                  a_uniform, e_small):
    """Key that switches a polynomial multiplying s_from into a pair under s_to.

    For digit j: component 1 is the uniform a_j; component 0 is
    b_j[m] = -a_j[m] s_to[m] + e_j[m] + [m in digit j] (P mod q_m) s_from[m]   (mod m)
    on all L+K limbs, evaluation domain.  s_*_eval are the secrets on all L+K moduli;
    a_uniform[j] are L+K uniform limbs; e_small[j] is a small signed polynomial."""
    all_ids = list(range(pr.L + pr.K))
    evk = []
    for j, dig in enumerate(pr.digits(pr.L)):
        e_eval = to_eval(pr, e_small[j], all_ids)
        b = []
        for m in all_ids:
            mod = pr.moduli[m]
            gadget = pr.P % mod if m in dig else 0
            b.append([(-a * st + e + gadget * sf) % mod
                      for a, st, e, sf in zip(a_uniform[j][m], s_to_eval[m], e_eval[m], s_from_eval[m])])
        evk.append([b, [list(x) for x in a_uniform[j]]])
    return evk


def phase(pr: Params, c0, c1, s_eval, ell: int) -> list[int]:
    """Decryption phase c0 + c1 s, CRT-reconstructed and centred modulo Q_ell, coefficient domain."""
    Q = pr.Q(ell)
    limbs = []
    for i in range(ell):
        qi = pr.q[i]
        ev = [(x + y * s) % qi for x, y, s in zip(c0[i], c1[i], s_eval[i])]
        limbs.append(intt(ev, qi, pr.psi[i]))
    out = []
    for n in range(pr.N):
        v = crt_reconstruct([limb[n] for limb in limbs], pr.q[:ell])
        out.append(v - Q if v > Q // 2 else v)
    return out


def poly_to_big(pr: Params, c_eval, ell: int) -> list[int]:
    """Evaluation-domain limbs -> centred big-integer coefficients modulo Q_ell."""
    Q = pr.Q(ell)
    limbs = [intt(c_eval[i], pr.q[i], pr.psi[i]) for i in range(ell)]
    out = []
    for n in range(pr.N):
        v = crt_reconstruct([limb[n] for limb in limbs], pr.q[:ell])
        out.append(v - Q if v > Q // 2 else v)
    return out
