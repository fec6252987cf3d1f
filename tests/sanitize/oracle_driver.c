/* Drives every entry point of the plain-C reference (oracle/ks_oracle.c, included below so that its static helpers are
 * instrumented too) on a small parameter set, for a build with -fsanitize=address,undefined: the point is that the
 * reference itself reads and writes nothing out of bounds and has no undefined arithmetic.  Also checks the transform
 * round trip and that a zero key gives a zero key-switch, so a miscompiled run does not pass silently.
 * Usage: oracle_driver logN L K dnum q_0 .. q_{L-1} p_0 .. p_{K-1} psi_0 .. psi_{L+K-1} */
#include "../../oracle/ks_oracle.c"

#include <stdio.h>

static u64 state = 0x243F6A8885A308D3ull;
static u64 next(void) { state ^= state >> 12; state ^= state << 25; state ^= state >> 27; return state * 0x2545F4914F6CDD1Dull; }
static void fill(u64 *a, size_t limbs, const u64 *mods, int nmods, u64 N) {
    for (size_t l = 0; l < limbs; l++)
        for (u64 n = 0; n < N; n++) a[l * N + n] = next() % mods[l % nmods];
}

int main(int argc, char **argv) {
    if (argc < 5) return 2;
    int logN = atoi(argv[1]), L = atoi(argv[2]), K = atoi(argv[3]), dnum = atoi(argv[4]);
    int M = L + K;
    if (argc != 5 + 2 * M) return 2;
    u64 *mods = malloc(sizeof(u64) * M), *psi = malloc(sizeof(u64) * M);
    for (int m = 0; m < M; m++) { mods[m] = strtoull(argv[5 + m], 0, 10); psi[m] = strtoull(argv[5 + M + m], 0, 10); }
    orc_ctx *c = orc_create(logN, L, K, dnum, mods, mods + L, psi);
    if (!c) return 3;
    u64 N = (u64)1 << logN;
    int fails = 0;
    for (int ell = 1; ell <= L; ell++) {
        int batch = 1 + ell % 2;
        /* transforms: round trip on the ciphertext limbs and one special limb */
        uint32_t ids[64];
        int nl = 0;
        for (int i = 0; i < ell; i++) ids[nl++] = (uint32_t)i;
        ids[nl++] = (uint32_t)(L + K - 1);
        u64 *x = malloc(sizeof(u64) * batch * nl * N), *y = malloc(sizeof(u64) * batch * nl * N);
        for (int b = 0; b < batch; b++)
            for (int l = 0; l < nl; l++)
                for (u64 n = 0; n < N; n++) x[((u64)b * nl + l) * N + n] = next() % mods[ids[l]];
        memcpy(y, x, sizeof(u64) * batch * nl * N);
        orc_ntt_fwd(c, y, ids, nl, batch);
        orc_ntt_inv(c, y, ids, nl, batch);
        if (memcmp(x, y, sizeof(u64) * batch * nl * N)) { printf("round trip differs at ell=%d\n", ell); fails++; }
        /* conversion from the first min(ell, 2) ciphertext limbs to everything else */
        int ns = ell < 2 ? 1 : 2;
        uint32_t src[2] = {0, 1}, dst[64];
        int nd = 0;
        for (int m = ns; m < M; m++) dst[nd++] = (uint32_t)m;
        u64 *bi = malloc(sizeof(u64) * batch * ns * N), *bo = malloc(sizeof(u64) * batch * nd * N);
        fill(bi, (size_t)batch * ns, mods, ns, N);
        orc_bconv(c, bi, src, ns, bo, dst, nd, batch);
        /* key-switch, with a random key and with the zero key */
        u64 *d = malloc(sizeof(u64) * batch * ell * N), *evk = malloc(sizeof(u64) * dnum * 2 * M * N);
        u64 *out = malloc(sizeof(u64) * batch * 2 * ell * N);
        fill(d, (size_t)batch * ell, mods, ell, N);
        fill(evk, (size_t)dnum * 2 * M, mods, M, N);
        orc_keyswitch(c, d, ell, evk, out, batch);
        memset(evk, 0, sizeof(u64) * dnum * 2 * M * N);
        orc_keyswitch(c, d, ell, evk, out, batch);
        for (u64 n = 0; n < (u64)batch * 2 * ell * N; n++)
            if (out[n]) { printf("zero key gives a non-zero result at ell=%d\n", ell); fails++; break; }
        fill(evk, (size_t)dnum * 2 * M, mods, M, N);
        /* rotations (hoisted, multiply-accumulate, two-level) */
        uint32_t gal[3] = {5, 25, 1};
        const u64 *keys[3] = {evk, evk, NULL};
        u64 *pt = malloc(sizeof(u64) * M * N);
        fill(pt, (size_t)M, mods, M, N);
        const u64 *pts[3] = {pt, NULL, pt};
        u64 *ct = malloc(sizeof(u64) * batch * 2 * ell * N), *rot = malloc(sizeof(u64) * batch * 2 * 2 * ell * N);
        fill(ct, (size_t)batch * 2 * ell, mods, ell, N);
        orc_rotate_hoisted(c, ct, ell, gal, keys, 2, rot, batch);
        orc_rotate_mac_hoisted(c, ct, ell, gal, keys, pts, 3, out, batch);
        const u64 *pts2[4] = {pt, NULL, NULL, pt};
        uint32_t giant[2] = {1, 25};
        const u64 *gkeys[2] = {NULL, evk};
        orc_bsgs_linear_transform(c, ct, ell, gal, keys, 2, giant, gkeys, 2, pts2, out, batch);
        /* multiplications */
        if (ell >= 2) {
            u64 *ctb = malloc(sizeof(u64) * batch * 2 * ell * N), *prod = malloc(sizeof(u64) * batch * 2 * (ell - 1) * N);
            fill(ctb, (size_t)batch * 2 * ell, mods, ell, N);
            orc_hmult_relin_rescale(c, ct, ctb, ell, evk, prod, batch);
            orc_hmult_relin_rescale_merged(c, ct, ctb, ell, evk, prod, batch);
            free(ctb); free(prod);
        }
        free(x); free(y); free(bi); free(bo); free(d); free(evk); free(out); free(pt); free(ct); free(rot);
    }
    orc_destroy(c);
    free(mods); free(psi);
    if (fails) return 1;
    printf("OK\n");
    return 0;
}
