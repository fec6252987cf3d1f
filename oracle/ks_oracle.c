/*
 * Reference tier (ii): the same algorithms as ckks_ref.py in plain C, for ring degrees where
 * pure Python is too slow.  TEST INFRASTRUCTURE ONLY: nothing in the product library includes,
 * links or calls this file, and it shares no source with the HIP path.
 *
 * Arithmetic is deliberately naive: every modular product is (unsigned __int128) a * b % m, the
 * transform is the textbook iterative radix-2 one, base conversion forms its sum term by term.
 * No Montgomery / Barrett / Shoup forms, no blocking, no fusion.  OpenMP only spreads independent
 * limbs over host cores.
 *
 * The paper names these operations without formulas (Background: "RNS and Limbs", "NTT",
 * "Evaluation Keys"; Motivation: hoisting; Kernel Code Generation: NTT, Base Conversion and
 * Elementwise kernel classes); definitions follow the cited textbook algorithms.  This tier is
 * pinned by tests that require identical output from the Python tier, which in turn is pinned by
 * brute force, CRT reconstruction and closed forms.
 *
 * Layouts (N contiguous everywhere): polynomial [limbs][N]; evaluation key [dnum][2][L+K][N]
 * (component 0 = b, 1 = a); ciphertext [2][ell][N].  Moduli index m: q_0..q_{L-1}, p_0..p_{K-1}.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;
typedef uint64_t u64;

static u64 mulmod(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
static u64 addmod(u64 a, u64 b, u64 m) { u64 s = a + b; return s >= m ? s - m : s; }
static u64 submod(u64 a, u64 b, u64 m) { return a >= b ? a - b : a + m - b; }

static u64 powmod(u64 a, u64 e, u64 m) {
    u64 r = 1 % m;
    a %= m;
    while (e) {
        if (e & 1) r = mulmod(r, a, m);
        a = mulmod(a, a, m);
        e >>= 1;
    }
    return r;
}
/* m prime */
static u64 invmod(u64 a, u64 m) { return powmod(a % m, m - 2, m); }

static uint32_t brv(uint32_t k, int bits) {
    uint32_t r = 0;
    for (int i = 0; i < bits; i++) { r = (r << 1) | (k & 1); k >>= 1; }
    return r;
}

typedef struct {
    int logN, L, K, dnum, alpha;
    u64 N;
    u64 *mod;   /* [L+K] */
    u64 *psi;   /* [L+K] */
    u64 **w;    /* [L+K][N]: psi^brv(k)      */
    u64 **winv; /* [L+K][N]: psi^-brv(k)     */
} orc_ctx;

orc_ctx *orc_create(int logN, int L, int K, int dnum, const u64 *q, const u64 *p, const u64 *psi) {
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->logN = logN; c->L = L; c->K = K; c->dnum = dnum;
    c->alpha = dnum > 0 ? (L + dnum - 1) / dnum : L;
    c->N = (u64)1 << logN;
    int M = L + K;
    c->mod = (u64 *)malloc(sizeof(u64) * M);
    c->psi = (u64 *)malloc(sizeof(u64) * M);
    c->w = (u64 **)malloc(sizeof(u64 *) * M);
    c->winv = (u64 **)malloc(sizeof(u64 *) * M);
    for (int m = 0; m < M; m++) {
        c->mod[m] = m < L ? q[m] : p[m - L];
        c->psi[m] = psi[m];
    }
#pragma omp parallel for schedule(dynamic)
    for (int m = 0; m < M; m++) {
        u64 mod = c->mod[m], N = c->N;
        u64 *pw = (u64 *)malloc(sizeof(u64) * N);
        c->w[m] = (u64 *)malloc(sizeof(u64) * N);
        c->winv[m] = (u64 *)malloc(sizeof(u64) * N);
        u64 ps = c->psi[m], psi_inv = invmod(ps, mod);
        pw[0] = 1;
        for (u64 i = 1; i < N; i++) pw[i] = mulmod(pw[i - 1], ps, mod);
        for (u64 k = 0; k < N; k++) c->w[m][k] = pw[brv((uint32_t)k, logN)];
        pw[0] = 1;
        for (u64 i = 1; i < N; i++) pw[i] = mulmod(pw[i - 1], psi_inv, mod);
        for (u64 k = 0; k < N; k++) c->winv[m][k] = pw[brv((uint32_t)k, logN)];
        free(pw);
    }
    return c;
}

void orc_destroy(orc_ctx *c) {
    if (!c) return;
    for (int m = 0; m < c->L + c->K; m++) { free(c->w[m]); free(c->winv[m]); }
    free(c->w); free(c->winv); free(c->mod); free(c->psi); free(c);
}

/* forward transform of one limb, in place: natural order in, bit-reversed order out */
static void ntt_limb(const orc_ctx *c, int m, u64 *a) {
    u64 mod = c->mod[m], N = c->N;
    for (u64 blocks = 1, half = N / 2; half >= 1; blocks *= 2, half /= 2) {
        for (u64 b = 0; b < blocks; b++) {
            u64 w = c->w[m][blocks + b];
            u64 lo = 2 * b * half;
            for (u64 j = lo; j < lo + half; j++) {
                u64 t = mulmod(a[j + half], w, mod);
                a[j + half] = submod(a[j], t, mod);
                a[j] = addmod(a[j], t, mod);
            }
        }
    }
}

/* inverse transform of one limb, in place: bit-reversed order in, natural order out */
static void intt_limb(const orc_ctx *c, int m, u64 *a) {
    u64 mod = c->mod[m], N = c->N;
    for (u64 blocks = N / 2, half = 1; blocks >= 1; blocks /= 2, half *= 2) {
        for (u64 b = 0; b < blocks; b++) {
            u64 w = c->winv[m][blocks + b];
            u64 lo = 2 * b * half;
            for (u64 j = lo; j < lo + half; j++) {
                u64 u = a[j], v = a[j + half];
                a[j] = addmod(u, v, mod);
                a[j + half] = mulmod(submod(u, v, mod), w, mod);
            }
        }
    }
    u64 ninv = invmod(N % mod, mod);
    for (u64 j = 0; j < N; j++) a[j] = mulmod(a[j], ninv, mod);
}

/* data: [batch][nlimbs][N]; mod_ids[nlimbs] index q|p */
void orc_ntt_fwd(const orc_ctx *c, u64 *data, const uint32_t *mod_ids, int nlimbs, int batch) {
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)nlimbs * batch; i++) ntt_limb(c, mod_ids[i % nlimbs], data + (u64)i * c->N);
}
void orc_ntt_inv(const orc_ctx *c, u64 *data, const uint32_t *mod_ids, int nlimbs, int batch) {
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)nlimbs * batch; i++) intt_limb(c, mod_ids[i % nlimbs], data + (u64)i * c->N);
}

/* Fast base conversion of one polynomial: in [n_src][N] coefficient domain -> out [n_dst][N].
 * out_t = sum_i [x_i (D/q_i)^-1]_{q_i} * (D/q_i)  mod t, D = product of the source moduli. */
static void bconv_poly(const orc_ctx *c, const u64 *in, const uint32_t *src, int n_src,
                       u64 *out, const uint32_t *dst, int n_dst) {
    u64 N = c->N;
    u64 *inv = (u64 *)malloc(sizeof(u64) * n_src);           /* (D/q_i)^-1 mod q_i */
    u64 *hat = (u64 *)malloc(sizeof(u64) * n_src * n_dst);    /* (D/q_i) mod t      */
    for (int i = 0; i < n_src; i++) {
        u64 qi = c->mod[src[i]], prod = 1;
        for (int k = 0; k < n_src; k++)
            if (k != i) prod = mulmod(prod, c->mod[src[k]] % qi, qi);
        inv[i] = invmod(prod, qi);
        for (int t = 0; t < n_dst; t++) {
            u64 mt = c->mod[dst[t]], pr = 1 % mt;
            for (int k = 0; k < n_src; k++)
                if (k != i) pr = mulmod(pr, c->mod[src[k]] % mt, mt);
            hat[i * n_dst + t] = pr;
        }
    }
    u64 *y = (u64 *)malloc(sizeof(u64) * n_src * N);
    for (int i = 0; i < n_src; i++) {
        u64 qi = c->mod[src[i]];
        for (u64 n = 0; n < N; n++) y[i * N + n] = mulmod(in[i * N + n], inv[i], qi);
    }
#pragma omp parallel for schedule(dynamic)
    for (int t = 0; t < n_dst; t++) {
        u64 mt = c->mod[dst[t]];
        for (u64 n = 0; n < N; n++) {
            u64 acc = 0;
            for (int i = 0; i < n_src; i++) acc = addmod(acc, mulmod(y[i * N + n] % mt, hat[i * n_dst + t], mt), mt);
            out[t * N + n] = acc;
        }
    }
    free(y); free(inv); free(hat);
}

void orc_bconv(const orc_ctx *c, const u64 *in, const uint32_t *src, int n_src,
               u64 *out, const uint32_t *dst, int n_dst, int batch) {
    for (int b = 0; b < batch; b++)
        bconv_poly(c, in + (u64)b * n_src * c->N, src, n_src, out + (u64)b * n_dst * c->N, dst, n_dst);
}

/* ------------------------------------------------------------------------------------------ */

static int ext_id(const orc_ctx *c, int ell, int pos) { return pos < ell ? pos : c->L + (pos - ell); }

/* Decompose and raise d [ell][N] (evaluation domain) to lifted [ndig][ell+K][N] (evaluation
 * domain), limb order q_0..q_{ell-1}, p_0..p_{K-1}.  Returns the digit count. */
static int mod_up(const orc_ctx *c, const u64 *d, int ell, u64 *lifted) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig = (ell + c->alpha - 1) / c->alpha;
    u64 *coeff = (u64 *)malloc(sizeof(u64) * ell * N);
    memcpy(coeff, d, sizeof(u64) * ell * N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ell; i++) intt_limb(c, i, coeff + (u64)i * N);
    for (int j = 0; j < ndig; j++) {
        int lo = j * c->alpha, hi = lo + c->alpha < ell ? lo + c->alpha : ell;
        int n_src = hi - lo, n_dst = E - n_src;
        uint32_t *src = (uint32_t *)malloc(sizeof(uint32_t) * n_src);
        uint32_t *dst = (uint32_t *)malloc(sizeof(uint32_t) * n_dst);
        int *dst_pos = (int *)malloc(sizeof(int) * n_dst);
        for (int i = 0; i < n_src; i++) src[i] = lo + i;
        int nd = 0;
        for (int pos = 0; pos < E; pos++) {
            if (pos >= lo && pos < hi) continue;
            dst[nd] = ext_id(c, ell, pos); dst_pos[nd] = pos; nd++;
        }
        u64 *conv = (u64 *)malloc(sizeof(u64) * n_dst * N);
        bconv_poly(c, coeff + (u64)lo * N, src, n_src, conv, dst, n_dst);
        u64 *Lj = lifted + (u64)j * E * N;
#pragma omp parallel for schedule(dynamic)
        for (int t = 0; t < n_dst; t++) {
            ntt_limb(c, dst[t], conv + (u64)t * N);
            memcpy(Lj + (u64)dst_pos[t] * N, conv + (u64)t * N, sizeof(u64) * N);
        }
        for (int i = lo; i < hi; i++) memcpy(Lj + (u64)i * N, d + (u64)i * N, sizeof(u64) * N);
        free(conv); free(src); free(dst); free(dst_pos);
    }
    free(coeff);
    return ndig;
}

/* acc [2][ell+K][N] = sum_j lifted_j * evk[j][c], evk [dnum][2][L+K][N] */
static void inner_product(const orc_ctx *c, const u64 *lifted, int ndig, int ell, const u64 *evk, u64 *acc) {
    u64 N = c->N;
    int E = ell + c->K, M = c->L + c->K;
#pragma omp parallel for schedule(dynamic)
    for (int idx = 0; idx < 2 * E; idx++) {
        int comp = idx / E, pos = idx % E;
        int m = ext_id(c, ell, pos);
        u64 mod = c->mod[m];
        u64 *row = acc + ((u64)comp * E + pos) * N;
        for (u64 n = 0; n < N; n++) row[n] = 0;
        for (int j = 0; j < ndig; j++) {
            const u64 *src = lifted + ((u64)j * E + pos) * N;
            const u64 *key = evk + (((u64)j * 2 + comp) * M + m) * N;
            for (u64 n = 0; n < N; n++) row[n] = addmod(row[n], mulmod(src[n], key[n], mod), mod);
        }
    }
}

/* Divide acc_c [ell+K][N] by P: out [ell][N] */
static void mod_down(const orc_ctx *c, const u64 *acc_c, int ell, u64 *out) {
    u64 N = c->N;
    int K = c->K;
    u64 *special = (u64 *)malloc(sizeof(u64) * K * N);
    memcpy(special, acc_c + (u64)ell * N, sizeof(u64) * K * N);
    uint32_t *src = (uint32_t *)malloc(sizeof(uint32_t) * K);
    uint32_t *dst = (uint32_t *)malloc(sizeof(uint32_t) * ell);
    for (int k = 0; k < K; k++) src[k] = c->L + k;
    for (int i = 0; i < ell; i++) dst[i] = i;
#pragma omp parallel for schedule(dynamic)
    for (int k = 0; k < K; k++) intt_limb(c, c->L + k, special + (u64)k * N);
    u64 *conv = (u64 *)malloc(sizeof(u64) * ell * N);
    bconv_poly(c, special, src, K, conv, dst, ell);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ell; i++) {
        u64 qi = c->mod[i];
        ntt_limb(c, i, conv + (u64)i * N);
        u64 Pmod = 1;
        for (int k = 0; k < K; k++) Pmod = mulmod(Pmod, c->mod[c->L + k] % qi, qi);
        u64 pinv = invmod(Pmod, qi);
        for (u64 n = 0; n < N; n++)
            out[(u64)i * N + n] = mulmod(submod(acc_c[(u64)i * N + n], conv[(u64)i * N + n], qi), pinv, qi);
    }
    free(special); free(conv); free(src); free(dst);
}

/* d [batch][ell][N], evk [dnum][2][L+K][N] -> out [batch][2][ell][N] */
void orc_keyswitch(const orc_ctx *c, const u64 *d, int ell, const u64 *evk, u64 *out, int batch) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig_max = (ell + c->alpha - 1) / c->alpha;
    u64 *lifted = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *acc = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    for (int b = 0; b < batch; b++) {
        int ndig = mod_up(c, d + (u64)b * ell * N, ell, lifted);
        inner_product(c, lifted, ndig, ell, evk, acc);
        for (int comp = 0; comp < 2; comp++)
            mod_down(c, acc + (u64)comp * E * N, ell, out + ((u64)b * 2 + comp) * ell * N);
    }
    free(lifted); free(acc);
}

/* sigma_g on one coefficient-domain limb: X^i -> +-X^(i g mod N) */
static void automorphism_coeff(const u64 *a, u64 *out, u64 N, u64 g, u64 mod) {
    for (u64 i = 0; i < N; i++) {
        u64 e = (i * g) % (2 * N);
        if (e < N) out[e] = a[i];
        else out[e - N] = a[i] ? mod - a[i] : 0;
    }
}

/* sigma_g on one evaluation-domain limb, by going through the coefficient domain */
static void sigma_eval(const orc_ctx *c, int m, const u64 *in, u64 *out, u64 g) {
    u64 N = c->N;
    u64 *tmp = (u64 *)malloc(sizeof(u64) * N);
    memcpy(tmp, in, sizeof(u64) * N);
    intt_limb(c, m, tmp);
    automorphism_coeff(tmp, out, N, g, c->mod[m]);
    ntt_limb(c, m, out);
    free(tmp);
}

/* ct [batch][2][ell][N]; galois[n_rot]; rot_keys[n_rot] -> out [batch][n_rot][2][ell][N].
 * One decompose-and-raise of c1 per ciphertext is shared by all rotations. */
void orc_rotate_hoisted(const orc_ctx *c, const u64 *ct, int ell, const uint32_t *galois,
                        const u64 *const *rot_keys, int n_rot, u64 *out, int batch) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig_max = (ell + c->alpha - 1) / c->alpha;
    u64 *lifted = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *rotated = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *acc = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    u64 *s0 = (u64 *)malloc(sizeof(u64) * ell * N);
    for (int b = 0; b < batch; b++) {
        const u64 *c0 = ct + (u64)b * 2 * ell * N, *c1 = c0 + (u64)ell * N;
        int ndig = mod_up(c, c1, ell, lifted);
        for (int r = 0; r < n_rot; r++) {
            u64 g = galois[r];
#pragma omp parallel for schedule(dynamic)
            for (int idx = 0; idx < ndig * E; idx++) {
                int pos = idx % E;
                sigma_eval(c, ext_id(c, ell, pos), lifted + (u64)idx * N, rotated + (u64)idx * N, g);
            }
            inner_product(c, rotated, ndig, ell, rot_keys[r], acc);
            u64 *o = out + (((u64)b * n_rot + r) * 2) * ell * N;
            for (int comp = 0; comp < 2; comp++) mod_down(c, acc + (u64)comp * E * N, ell, o + (u64)comp * ell * N);
#pragma omp parallel for schedule(dynamic)
            for (int i = 0; i < ell; i++) {
                sigma_eval(c, i, c0 + (u64)i * N, s0 + (u64)i * N, g);
                u64 qi = c->mod[i];
                for (u64 n = 0; n < N; n++) o[(u64)i * N + n] = addmod(o[(u64)i * N + n], s0[(u64)i * N + n], qi);
            }
        }
    }
    free(lifted); free(rotated); free(acc); free(s0);
}

/* One rotated ciphertext on the extended basis before any division by P: term = (acc_0 + P sigma_g(c0), acc_1), acc the
 * inner product of the sigma_g-permuted raised digits of c1 with the rotation key.  g = 1 is the unrotated ciphertext:
 * no key, term = P (c0, c1) on the ciphertext limbs and 0 on the special limbs.  `rotated`: scratch [ndig][E][N]. */
static void rotation_term(const orc_ctx *c, const u64 *c0, const u64 *c1, const u64 *lifted, int ndig, int ell, u64 g,
                          const u64 *key, u64 *rotated, u64 *term) {
    u64 N = c->N;
    int E = ell + c->K;
    if (g == 1) {
        memset(term, 0, sizeof(u64) * 2 * E * N);
        for (int i = 0; i < ell; i++) {
            u64 qi = c->mod[i], Pmod = 1;
            for (int k = 0; k < c->K; k++) Pmod = mulmod(Pmod, c->mod[c->L + k] % qi, qi);
            for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) {
                term[n] = mulmod(Pmod, c0[n], qi);
                term[(u64)E * N + n] = mulmod(Pmod, c1[n], qi);
            }
        }
        return;
    }
#pragma omp parallel for schedule(dynamic)
    for (int idx = 0; idx < ndig * E; idx++) {
        int pos = idx % E;
        sigma_eval(c, ext_id(c, ell, pos), lifted + (u64)idx * N, rotated + (u64)idx * N, g);
    }
    inner_product(c, rotated, ndig, ell, key, term);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ell; i++) {
        u64 qi = c->mod[i], Pmod = 1;
        for (int k = 0; k < c->K; k++) Pmod = mulmod(Pmod, c->mod[c->L + k] % qi, qi);
        u64 *s0 = (u64 *)malloc(sizeof(u64) * N);
        sigma_eval(c, i, c0 + (u64)i * N, s0, g);
        for (u64 n = 0; n < N; n++) term[(u64)i * N + n] = addmod(term[(u64)i * N + n], mulmod(Pmod, s0[n], qi), qi);
        free(s0);
    }
}

/* u (+)= sum_r pt_r * rotation_term(ct, g_r): the inner sum of a baby-step giant-step transform on the extended basis.
 * pts[r] holds all L + K limbs in evaluation domain, like a key component; NULL = the constant 1. */
static void rotate_mac_sum(const orc_ctx *c, const u64 *c0, const u64 *c1, int ell, const uint32_t *galois,
                           const u64 *const *rot_keys, const u64 *const *pts, int n_rot, u64 *lifted, u64 *rotated, u64 *term,
                           u64 *u) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig = mod_up(c, c1, ell, lifted);
    for (int r = 0; r < n_rot; r++) {
        rotation_term(c, c0, c1, lifted, ndig, ell, galois[r], rot_keys[r], rotated, term);
#pragma omp parallel for schedule(dynamic)
        for (int idx = 0; idx < 2 * E; idx++) {
            int pos = idx % E, m = ext_id(c, ell, pos);
            u64 mod = c->mod[m];
            const u64 *pt = pts[r] ? pts[r] + (u64)m * N : NULL;
            u64 *t = term + (u64)idx * N, *ui = u + (u64)idx * N;
            for (u64 n = 0; n < N; n++) ui[n] = addmod(ui[n], pt ? mulmod(pt[n], t[n], mod) : t[n], mod);
        }
    }
}

/* Double-hoisted rotate-multiply-accumulate: out = mod_down(sum_r pt_r * rotation_term(ct, g_r)). */
void orc_rotate_mac_hoisted(const orc_ctx *c, const u64 *ct, int ell, const uint32_t *galois,
                            const u64 *const *rot_keys, const u64 *const *pts, int n_rot, u64 *out, int batch) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig_max = (ell + c->alpha - 1) / c->alpha;
    u64 *lifted = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *rotated = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *term = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    for (int b = 0; b < batch; b++) {
        const u64 *c0 = ct + (u64)b * 2 * ell * N, *c1 = c0 + (u64)ell * N;
        memset(u, 0, sizeof(u64) * 2 * E * N);
        rotate_mac_sum(c, c0, c1, ell, galois, rot_keys, pts, n_rot, lifted, rotated, term, u);
        u64 *o = out + (u64)b * 2 * ell * N;
        for (int comp = 0; comp < 2; comp++) mod_down(c, u + (u64)comp * E * N, ell, o + (u64)comp * ell * N);
    }
    free(lifted); free(rotated); free(term); free(u);
}

/* Baby-step giant-step linear transform, double-hoisted at both levels:
 * out = mod_down(sum_g rotation_term(v_g, G_g)),  v_g = mod_down(sum_b pts[g * n1 + b] * rotation_term(ct, B_b)). */
void orc_bsgs_linear_transform(const orc_ctx *c, const u64 *ct, int ell, const uint32_t *baby_galois,
                               const u64 *const *baby_keys, int n1, const uint32_t *giant_galois,
                               const u64 *const *giant_keys, int n2, const u64 *const *pts, u64 *out, int batch) {
    u64 N = c->N;
    int E = ell + c->K;
    int ndig_max = (ell + c->alpha - 1) / c->alpha;
    u64 *lifted = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *rotated = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *term = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    u64 *uo = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    u64 *v = (u64 *)malloc(sizeof(u64) * 2 * ell * N);
    for (int b = 0; b < batch; b++) {
        const u64 *c0 = ct + (u64)b * 2 * ell * N, *c1 = c0 + (u64)ell * N;
        memset(uo, 0, sizeof(u64) * 2 * E * N);
        for (int g = 0; g < n2; g++) {
            memset(u, 0, sizeof(u64) * 2 * E * N);
            rotate_mac_sum(c, c0, c1, ell, baby_galois, baby_keys, pts + (u64)g * n1, n1, lifted, rotated, term, u);
            for (int comp = 0; comp < 2; comp++) mod_down(c, u + (u64)comp * E * N, ell, v + (u64)comp * ell * N);
            const u64 *one_pt = NULL;
            rotate_mac_sum(c, v, v + (u64)ell * N, ell, giant_galois + g, giant_keys + g, &one_pt, 1, lifted, rotated, term, uo);
        }
        u64 *o = out + (u64)b * 2 * ell * N;
        for (int comp = 0; comp < 2; comp++) mod_down(c, uo + (u64)comp * E * N, ell, o + (u64)comp * ell * N);
    }
    free(lifted); free(rotated); free(term); free(u); free(uo); free(v);
}

static void rescale_poly(const orc_ctx *c, const u64 *poly, int ell, u64 *out) {
    u64 N = c->N;
    u64 ql = c->mod[ell - 1], half = (ql - 1) / 2;
    u64 *r = (u64 *)malloc(sizeof(u64) * N);
    memcpy(r, poly + (u64)(ell - 1) * N, sizeof(u64) * N);
    intt_limb(c, ell - 1, r);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ell - 1; i++) {
        u64 qi = c->mod[i];
        u64 *w = (u64 *)malloc(sizeof(u64) * N);
        for (u64 n = 0; n < N; n++) {
            u64 x = r[n] % qi;
            w[n] = r[n] > half ? submod(x, ql % qi, qi) : x;   /* centred remainder, reduced mod q_i */
        }
        ntt_limb(c, i, w);
        u64 qlinv = invmod(ql % qi, qi);
        for (u64 n = 0; n < N; n++)
            out[(u64)i * N + n] = mulmod(submod(poly[(u64)i * N + n], w[n], qi), qlinv, qi);
        free(w);
    }
    free(r);
}

/* cta, ctb [batch][2][ell][N] (component 0 = b, 1 = a); rlk as evk -> out [batch][2][ell-1][N] */
void orc_hmult_relin_rescale(const orc_ctx *c, const u64 *cta, const u64 *ctb, int ell,
                             const u64 *rlk, u64 *out, int batch) {
    u64 N = c->N;
    u64 sz = (u64)ell * N;
    u64 *d0 = (u64 *)malloc(sizeof(u64) * sz), *d1 = (u64 *)malloc(sizeof(u64) * sz), *d2 = (u64 *)malloc(sizeof(u64) * sz);
    u64 *ks = (u64 *)malloc(sizeof(u64) * 2 * sz);
    for (int b = 0; b < batch; b++) {
        const u64 *b1 = cta + (u64)b * 2 * sz, *a1 = b1 + sz;
        const u64 *b2 = ctb + (u64)b * 2 * sz, *a2 = b2 + sz;
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < ell; i++) {
            u64 qi = c->mod[i];
            for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) {
                d0[n] = mulmod(b1[n], b2[n], qi);
                d1[n] = addmod(mulmod(a1[n], b2[n], qi), mulmod(a2[n], b1[n], qi), qi);
                d2[n] = mulmod(a1[n], a2[n], qi);
            }
        }
        orc_keyswitch(c, d2, ell, rlk, ks, 1);
        for (int i = 0; i < ell; i++) {
            u64 qi = c->mod[i];
            for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) {
                d0[n] = addmod(d0[n], ks[n], qi);
                d1[n] = addmod(d1[n], ks[sz + n], qi);
            }
        }
        u64 *o = out + (u64)b * 2 * (ell - 1) * N;
        rescale_poly(c, d0, ell, o);
        rescale_poly(c, d1, ell, o + (u64)(ell - 1) * N);
    }
    free(d0); free(d1); free(d2); free(ks);
}

/* ModDown merged with the rescale that follows (Compiler: "mod down merging"): acc' = acc + P * addend on the
 * ciphertext limbs, then one division by D = P * q_{ell-1} through a fast conversion from the basis
 * {p_0..p_{K-1}, q_{ell-1}} to q_0..q_{ell-2}.  Floor-type: every coefficient is floor(acc' / D) - u, 0 <= u <= K. */
static void mod_down_merged(const orc_ctx *c, const u64 *acc_c, const u64 *addend, int ell, u64 *out) {
    u64 N = c->N;
    int K = c->K, S = K + 1;
    u64 *accp = (u64 *)malloc(sizeof(u64) * ell * N);
    for (int i = 0; i < ell; i++) {
        u64 qi = c->mod[i], Pmod = 1;
        for (int k = 0; k < K; k++) Pmod = mulmod(Pmod, c->mod[c->L + k] % qi, qi);
        for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) accp[n] = addmod(acc_c[n], mulmod(Pmod, addend[n], qi), qi);
    }
    u64 *srcl = (u64 *)malloc(sizeof(u64) * S * N);
    memcpy(srcl, acc_c + (u64)ell * N, sizeof(u64) * K * N);
    memcpy(srcl + (u64)K * N, accp + (u64)(ell - 1) * N, sizeof(u64) * N);
    uint32_t *src = (uint32_t *)malloc(sizeof(uint32_t) * S);
    uint32_t *dst = (uint32_t *)malloc(sizeof(uint32_t) * ell);
    for (int k = 0; k < K; k++) src[k] = c->L + k;
    src[K] = ell - 1;
    for (int i = 0; i < ell - 1; i++) dst[i] = i;
#pragma omp parallel for schedule(dynamic)
    for (int k = 0; k < S; k++) intt_limb(c, src[k], srcl + (u64)k * N);
    u64 *conv = (u64 *)malloc(sizeof(u64) * ell * N);
    bconv_poly(c, srcl, src, S, conv, dst, ell - 1);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ell - 1; i++) {
        u64 qi = c->mod[i];
        ntt_limb(c, i, conv + (u64)i * N);
        u64 Dmod = c->mod[ell - 1] % qi;
        for (int k = 0; k < K; k++) Dmod = mulmod(Dmod, c->mod[c->L + k] % qi, qi);
        u64 dinv = invmod(Dmod, qi);
        for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) out[n] = mulmod(submod(accp[n], conv[n], qi), dinv, qi);
    }
    free(accp); free(srcl); free(conv); free(src); free(dst);
}

void orc_hmult_relin_rescale_merged(const orc_ctx *c, const u64 *cta, const u64 *ctb, int ell,
                                    const u64 *rlk, u64 *out, int batch) {
    u64 N = c->N;
    u64 sz = (u64)ell * N;
    int E = ell + c->K;
    int ndig_max = (ell + c->alpha - 1) / c->alpha;
    u64 *d0 = (u64 *)malloc(sizeof(u64) * sz), *d1 = (u64 *)malloc(sizeof(u64) * sz), *d2 = (u64 *)malloc(sizeof(u64) * sz);
    u64 *lifted = (u64 *)malloc(sizeof(u64) * ndig_max * E * N);
    u64 *acc = (u64 *)malloc(sizeof(u64) * 2 * E * N);
    for (int b = 0; b < batch; b++) {
        const u64 *b1 = cta + (u64)b * 2 * sz, *a1 = b1 + sz;
        const u64 *b2 = ctb + (u64)b * 2 * sz, *a2 = b2 + sz;
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < ell; i++) {
            u64 qi = c->mod[i];
            for (u64 n = (u64)i * N; n < (u64)(i + 1) * N; n++) {
                d0[n] = mulmod(b1[n], b2[n], qi);
                d1[n] = addmod(mulmod(a1[n], b2[n], qi), mulmod(a2[n], b1[n], qi), qi);
                d2[n] = mulmod(a1[n], a2[n], qi);
            }
        }
        int ndig = mod_up(c, d2, ell, lifted);
        inner_product(c, lifted, ndig, ell, rlk, acc);
        u64 *o = out + (u64)b * 2 * (ell - 1) * N;
        mod_down_merged(c, acc, d0, ell, o);
        mod_down_merged(c, acc + (u64)E * N, d1, ell, o + (u64)(ell - 1) * N);
    }
    free(d0); free(d1); free(d2); free(lifted); free(acc);
}

int orc_max_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
