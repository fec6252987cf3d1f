// Context construction: parameter validation, twiddle tables, base-conversion constants.
// Host-side number theory here is the library's own (128-bit products); it shares nothing with
// the CPU reference used by the tests.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <string>

#include "ks_internal.hpp"

namespace ks {

typedef unsigned __int128 u128;

uint64_t h_mulmod(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)((u128)a * b % m); }

uint64_t h_powmod(uint64_t a, uint64_t e, uint64_t m) {
    uint64_t r = 1 % m;
    a %= m;
    for (; e; e >>= 1) {
        if (e & 1) r = h_mulmod(r, a, m);
        a = h_mulmod(a, a, m);
    }
    return r;
}

uint64_t h_invmod(uint64_t a, uint64_t m) { return h_powmod(a % m, m - 2, m); }  // m prime

static bool h_is_prime(uint64_t n) {
    if (n < 2) return false;
    static const uint64_t bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (uint64_t b : bases) {
        if (n % b == 0) return n == b;
    }
    uint64_t d = n - 1;
    int s = 0;
    while ((d & 1) == 0) { d >>= 1; ++s; }
    for (uint64_t b : bases) {
        uint64_t x = h_powmod(b, d, n);
        if (x == 1 || x == n - 1) continue;
        bool comp = true;
        for (int i = 1; i < s; ++i) {
            x = h_mulmod(x, x, n);
            if (x == n - 1) { comp = false; break; }
        }
        if (comp) return false;
    }
    return true;
}

// Smallest primitive 2N-th root of unity modulo the prime m (m = 1 mod 2N): the N candidates are the odd
// powers of any one of them.
static uint64_t h_minimal_psi(uint64_t m, uint32_t N) {
    uint64_t root = 0;
    for (uint64_t x = 2;; ++x) {
        root = h_powmod(x, (m - 1) / (2ull * N), m);
        if (h_powmod(root, N, m) == m - 1) break;
    }
    const uint64_t sq = h_mulmod(root, root, m);
    uint64_t best = root, cur = root;
    for (uint32_t i = 1; i < N; ++i) {
        cur = h_mulmod(cur, sq, m);
        best = std::min(best, cur);
    }
    return best;
}

static uint32_t h_brv(uint32_t k, uint32_t bits) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < bits; ++i) { r = (r << 1) | (k & 1); k >>= 1; }
    return r;
}

static Mod make_mod(uint64_t m) { return Mod{(double)m, 1.0 / (double)m}; }

void fill_bconv_plan(const ks_ctx* c, BConvPlan* plan, const uint32_t* src_ids, const uint16_t* src_limb, uint32_t n_src,
                     const uint32_t* dst_ids, const uint16_t* dst_limb, uint32_t n_dst, uint32_t shape_src) {
    memset(plan, 0, sizeof(BConvPlan));
    if (shape_src < n_src) shape_src = n_src;
    plan->n_src = n_src;
    plan->n_dst = n_dst;
    plan->mfma_nm = (shape_src + 5) / 6;
    plan->mfma_nps = (shape_src + 2 * plan->mfma_nm - 1) / (2 * plan->mfma_nm);
    for (uint32_t k = 0; k < (uint32_t)kMfmaSlots * 3; ++k) plan->mfma_src_limb[k] = src_limb[k < n_src ? k : 0];
    for (uint32_t i = 0; i < n_src; ++i) {
        const uint64_t si = c->mod[src_ids[i]];
        uint64_t prod = 1;
        for (uint32_t k = 0; k < n_src; ++k)
            if (k != i) prod = h_mulmod(prod, c->mod[src_ids[k]] % si, si);
        plan->src_limb[i] = src_limb[i];
        plan->src_mod[i] = make_mod(si);
        plan->src_inv[i] = (double)h_invmod(prod, si);
    }
    // padding sources: factor 0 (from the memset) and the first real source's limb, so that kernels may run their
    // source loop past n_src without branching and still read valid numbers
    for (uint32_t i = n_src; i < (uint32_t)kMaxSrc; ++i) plan->src_limb[i] = src_limb[0];
    for (uint32_t t = 0; t < n_dst; ++t) {
        const uint64_t mt = c->mod[dst_ids[t]];
        plan->dst_limb[t] = dst_limb[t];
        plan->dst_mod[t] = make_mod(mt);
        plan->dst_mod_id[t] = (uint8_t)dst_ids[t];
        plan->trec[t].m = plan->dst_mod[t];
        plan->trec[t].mod_id = dst_ids[t];
        plan->trec[t].limb = dst_limb[t];
        for (uint32_t i = 0; i < n_src; ++i) {
            uint64_t prod = 1 % mt;
            for (uint32_t k = 0; k < n_src; ++k)
                if (k != i) prod = h_mulmod(prod, c->mod[src_ids[k]] % mt, mt);
            // factors against the pieces of a source residue: cut at 12 and 24 bits, or at 16 bits when every modulus is
            // below 2^32 (split3 / split2)
            const int cut = c->pieces == 2 ? 16 : 12;
            for (int k = 0; k < 3; ++k) {
                const uint64_t f = h_mulmod(prod, (1ull << (cut * k)) % mt, mt);
                const double centred = f > mt / 2 ? -(double)(mt - f) : (double)f;
                plan->hats[t][i][k] = k < c->pieces ? ldexp(centred, -cut * k) : 0.0;
            }
            plan->hat3[t][i][0] = (double)(prod & 0xFFFu);
            plan->hat3[t][i][1] = (double)((prod >> 12) & 0xFFFu);
            plan->hat3[t][i][2] = (double)(prod >> 24);
            // matrix-core operand rows: digit b of centred([(D / s_i) 256^a]_t), at the byte that pairs with digit a of source i
            const uint32_t slot = i / plan->mfma_nps, e = i % plan->mfma_nps;
            for (int a = 0; a < kMfmaPlanes; ++a) {
                const uint64_t f = h_mulmod(prod, (1ull << (8 * a)) % mt, mt);
                int64_t v = f > mt / 2 ? -(int64_t)(mt - f) : (int64_t)f;
                for (int b = 0; b < kMfmaPlanes; ++b) {
                    int64_t digit = b + 1 < kMfmaPlanes ? ((v + 128) & 255) - 128 : v;   // the last digit takes what is left (|.| <= 9)
                    v = (v - digit) / 256;
                    plan->afac[t][b][slot][a < 4 ? 4 * e + a : 12 + e] = (int8_t)digit;
                }
            }
        }
    }
}

hipError_t upload_plans(const BConvPlan* host_plans, uint32_t n_plans, uint32_t shape_src, PlanSet* out) {
    *out = PlanSet{};
    if (n_plans == 0 || n_plans > (uint32_t)kMaxDigits) return hipErrorInvalidValue;
    hipError_t e = hipMalloc(&out->d_plans, sizeof(BConvPlan) * n_plans);
    if (e != hipSuccess) return e;
    e = hipMemcpy(out->d_plans, host_plans, sizeof(BConvPlan) * n_plans, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(out->d_plans);
        out->d_plans = nullptr;
        return e;
    }
    out->n_plans = n_plans;
    out->shape_src = shape_src;
    for (uint32_t j = 0; j < n_plans; ++j) {
        out->max_targets = std::max(out->max_targets, host_plans[j].n_dst);
        out->meta.plan[j].n_dst = host_plans[j].n_dst;
        for (int k = 0; k < kMfmaSlots * 3; ++k) out->meta.plan[j].src_limb[k] = host_plans[j].mfma_src_limb[k];
    }
    return hipSuccess;
}

static thread_local std::string g_hip_error;
void set_hip_error(hipError_t e, const char* where) {
    g_hip_error = std::string(where) + ": " + hipGetErrorString(e);
}

}  // namespace ks

using namespace ks;

#define CK(call)                                   \
    do {                                           \
        hipError_t e_ = (call);                    \
        if (e_ != hipSuccess) {                    \
            set_hip_error(e_, #call);              \
            rc = KS_EHIP;                          \
            goto fail;                             \
        }                                          \
    } while (0)

extern "C" const char* ks_last_hip_error(void) { return ks::g_hip_error.c_str(); }

extern "C" const char* ks_strerror(int code) {
    switch (code) {
        case KS_OK: return "ok";
        case KS_EINVAL: return "invalid argument";
        case KS_EWORKSPACE: return "workspace missing or too small";
        case KS_EHIP: return "HIP runtime error (see ks_last_hip_error)";
        case KS_ENOMEM: return "out of memory";
        case KS_ENOTPREPARED: return "conversion not registered (call bconv_prepare first)";
        default: return "unknown error code";
    }
}

extern "C" int ks_ctx_set_option(ks_ctx* c, int option, int value) {
    if (!c) return KS_EINVAL;
    switch (option) {
        case KS_OPT_BCONV_TARGETS:
            if (value < 0 || value > 4) return KS_EINVAL;
            break;
        case KS_OPT_BCONV_KERNEL:
            if (value < 0 || value > 2) return KS_EINVAL;
            break;
        default: return KS_EINVAL;
    }
    c->opt[option] = value;
    return KS_OK;
}

extern "C" int ks_ctx_destroy(ks_ctx* c) {
    if (!c) return KS_EINVAL;
    (void)hipSetDevice(c->device);
    (void)hipFree(c->d_mod);
    (void)hipFree(c->d_ninv);
    (void)hipFree(c->d_Pinv);
    (void)hipFree(c->d_Pmod);
    (void)hipFree(c->d_one);
    (void)hipFree(c->d_moddown_scale);
    (void)hipFree(c->d_tw_fwd);
    (void)hipFree(c->d_tw_inv);
    (void)hipFree(c->d_trow);
    (void)hipFree(c->d_w16);
    for (auto& lv : c->levels) {
        (void)hipFree(lv.modup.d_plans);
        (void)hipFree(lv.moddown.d_plans);
        (void)hipFree(lv.d_qlinv);
        (void)hipFree(lv.d_modup_scale);
        (void)hipFree(lv.merged.d_plans);
        (void)hipFree(lv.d_merged_scale);
        (void)hipFree(lv.d_Dinv);
    }
    for (auto& kv : c->bconv_cache) (void)hipFree(kv.second.d_plans);
    delete c;
    return KS_OK;
}

extern "C" int ks_ctx_create(ks_ctx** out, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                             const uint64_t* q, const uint64_t* p, const uint64_t* psi, int device) {
    if (!out) return KS_EINVAL;
    *out = nullptr;
    if (logN < 12 || logN > 16) return KS_EINVAL;
    if (L == 0 || !q || (K > 0 && !p) || L + K > 255 || dnum == 0 || dnum > L) return KS_EINVAL;
    const uint32_t N = 1u << logN, M = L + K;
    const uint32_t alpha = (L + dnum - 1) / dnum;
    if (K > (uint32_t)kMaxSrc) return KS_EINVAL;
    if (K > 0 && alpha > (uint32_t)kMaxSrc) return KS_EINVAL;
    if ((L + alpha - 1) / alpha > (uint32_t)kMaxDigits) return KS_EINVAL;
    if (K > 0 && ((L + alpha - 1) / alpha) * M > (uint32_t)kMaxLimbs) return KS_EINVAL;

    ks_ctx* c = new (std::nothrow) ks_ctx;
    if (!c) return KS_ENOMEM;
    int rc = KS_OK;
    c->device = device;
    c->logN = logN; c->N = N; c->L = L; c->K = K; c->dnum = dnum; c->alpha = alpha; c->M = M;
    c->mod.resize(M);
    c->psi.resize(M);
    for (uint32_t m = 0; m < M; ++m) {
        const uint64_t v = m < L ? q[m] : p[m - L];
        if (v >= (1ull << 36) || v % (2ull * N) != 1 || !h_is_prime(v)) { rc = KS_EINVAL; goto fail; }
        for (uint32_t k = 0; k < m; ++k)
            if (c->mod[k] == v) { rc = KS_EINVAL; goto fail; }
        c->mod[m] = v;
        if (psi) {
            if (psi[m] == 0 || psi[m] >= v || h_powmod(psi[m], N, v) != v - 1) { rc = KS_EINVAL; goto fail; }
            c->psi[m] = psi[m];
        } else {
            c->psi[m] = h_minimal_psi(v, N);
        }
    }
    c->pieces = 2;
    for (uint64_t v : c->mod)
        if (v >> 32) c->pieces = 3;
    {
        CK(hipSetDevice(device));
        CK(bind_static_scratch(device));
        // per-modulus constants
        std::vector<Mod> hm(M);
        std::vector<double> hn(M), hP(L), hPm(L);
        for (uint32_t m = 0; m < M; ++m) {
            hm[m] = Mod{(double)c->mod[m], 1.0 / (double)c->mod[m]};
            hn[m] = (double)h_invmod(N % c->mod[m], c->mod[m]);
        }
        for (uint32_t i = 0; i < L; ++i) {
            uint64_t P = 1;
            for (uint32_t k = 0; k < K; ++k) P = h_mulmod(P, c->mod[L + k] % c->mod[i], c->mod[i]);
            hP[i] = (double)h_invmod(P, c->mod[i]);
            hPm[i] = (double)P;
        }
        CK(hipMalloc(&c->d_mod, sizeof(Mod) * M));
        CK(hipMalloc(&c->d_ninv, sizeof(double) * M));
        CK(hipMalloc(&c->d_Pinv, sizeof(double) * L));
        CK(hipMemcpy(c->d_mod, hm.data(), sizeof(Mod) * M, hipMemcpyHostToDevice));
        CK(hipMemcpy(c->d_ninv, hn.data(), sizeof(double) * M, hipMemcpyHostToDevice));
        CK(hipMemcpy(c->d_Pinv, hP.data(), sizeof(double) * L, hipMemcpyHostToDevice));
        CK(hipMalloc(&c->d_Pmod, sizeof(double) * L));
        {
            const uint64_t ones[2] = {1, 1};
            CK(hipMalloc(&c->d_one, sizeof(ones)));
            CK(hipMemcpy(c->d_one, ones, sizeof(ones), hipMemcpyHostToDevice));
        }
        CK(hipMemcpy(c->d_Pmod, hPm.data(), sizeof(double) * L, hipMemcpyHostToDevice));
        if (K > 0) {
            std::vector<double> sc(K);
            for (uint32_t k = 0; k < K; ++k) {
                const uint64_t pk = c->mod[L + k];
                uint64_t prod = 1;
                for (uint32_t k2 = 0; k2 < K; ++k2)
                    if (k2 != k) prod = h_mulmod(prod, c->mod[L + k2] % pk, pk);
                sc[k] = (double)h_mulmod(h_invmod(prod, pk), h_invmod(N % pk, pk), pk);
            }
            CK(hipMalloc(&c->d_moddown_scale, sizeof(double) * K));
            CK(hipMemcpy(c->d_moddown_scale, sc.data(), sizeof(double) * K, hipMemcpyHostToDevice));
        }

        // twiddle tables: W[k] = psi^brv(k), Winv[k] = psi^-brv(k)
        CK(hipMalloc(&c->d_tw_fwd, sizeof(double) * (size_t)M * N));
        CK(hipMalloc(&c->d_tw_inv, sizeof(double) * (size_t)M * N));
        CK(hipMalloc(&c->d_trow, sizeof(double) * 2 * (size_t)M * (N / 16)));
        CK(hipMalloc(&c->d_w16, sizeof(double) * 2 * (size_t)M * 8));
        c->tw_fwd = TwTables{c->d_tw_fwd, c->d_trow, c->d_w16};
        c->tw_inv = TwTables{c->d_tw_inv, c->d_trow + (size_t)M * (N / 16), c->d_w16 + (size_t)M * 8};
        std::vector<uint64_t> pw(N);
        std::vector<double> tab(N), trow(N / 16), w16(8);
        for (uint32_t m = 0; m < M; ++m) {
            const uint64_t mod = c->mod[m];
            for (int dir = 0; dir < 2; ++dir) {
                const uint64_t base = dir == 0 ? c->psi[m] : h_invmod(c->psi[m], mod);
                pw[0] = 1;
                for (uint32_t i = 1; i < N; ++i) pw[i] = h_mulmod(pw[i - 1], base, mod);
                for (uint32_t k = 0; k < N; ++k) tab[k] = (double)pw[h_brv(k, logN)];
                double* dst = (dir == 0 ? c->d_tw_fwd : c->d_tw_inv) + (size_t)m * N;
                CK(hipMemcpy(dst, tab.data(), sizeof(double) * N, hipMemcpyHostToDevice));
                // compact tables for the row kernels: last-pass generators and the powers of the 16th root of unity
                for (uint32_t i = 0; i < N / 16; ++i) trow[i] = tab[8 * (N / 16 + i)];
                for (uint32_t e = 0; e < 8; ++e) w16[e] = (double)pw[(size_t)(N / 8) * e];
                const TwTables& tt = dir == 0 ? c->tw_fwd : c->tw_inv;
                CK(hipMemcpy(const_cast<double*>(tt.trow) + (size_t)m * (N / 16), trow.data(), sizeof(double) * (N / 16),
                             hipMemcpyHostToDevice));
                CK(hipMemcpy(const_cast<double*>(tt.w16) + (size_t)m * 8, w16.data(), sizeof(double) * 8, hipMemcpyHostToDevice));
            }
        }

        // per-level pipeline tables (only meaningful with special primes)
        c->levels.resize(L);
        for (uint32_t ell = 1; ell <= L && K > 0; ++ell) {
            Level& lv = c->levels[ell - 1];
            lv.ell = ell;
            lv.E = ell + K;
            lv.ndig = (ell + alpha - 1) / alpha;
            auto ext_id = [&](uint32_t pos) { return pos < ell ? pos : L + (pos - ell); };
            std::vector<BConvPlan> plans(lv.ndig);
            lv.lifted_map.n = 0;
            const uint32_t max_src = std::min(alpha, ell);
            for (uint32_t j = 0; j < lv.ndig; ++j) {
                const uint32_t lo = j * alpha, hi = std::min(lo + alpha, ell);
                lv.digit_lo[j] = lo;
                lv.digit_hi[j] = hi;
                uint32_t src_ids[kMaxSrc];
                uint16_t src_limb[kMaxSrc];
                std::vector<uint32_t> dst_ids;
                std::vector<uint16_t> dst_limb;
                for (uint32_t i = lo; i < hi; ++i) { src_ids[i - lo] = i; src_limb[i - lo] = (uint16_t)i; }
                for (uint32_t pos = 0; pos < lv.E; ++pos) {
                    if (pos >= lo && pos < hi) continue;
                    dst_ids.push_back(ext_id(pos));
                    dst_limb.push_back((uint16_t)(j * lv.E + pos));
                    lv.lifted_map.off[lv.lifted_map.n] = (uint16_t)(j * lv.E + pos);
                    lv.lifted_map.mod[lv.lifted_map.n] = (uint8_t)ext_id(pos);
                    lv.lifted_map.n++;
                }
                fill_bconv_plan(c, &plans[j], src_ids, src_limb, hi - lo, dst_ids.data(), dst_limb.data(),
                                (uint32_t)dst_ids.size(), max_src);
            }
            lv.n_new = lv.lifted_map.n;
            {
                std::vector<double> sc(ell);
                for (uint32_t j = 0; j < lv.ndig; ++j) {
                    for (uint32_t i = lv.digit_lo[j]; i < lv.digit_hi[j]; ++i) {
                        const uint64_t qi = c->mod[i];
                        const uint64_t dinv = (uint64_t)plans[j].src_inv[i - lv.digit_lo[j]];
                        sc[i] = (double)h_mulmod(dinv, h_invmod(N % qi, qi), qi);
                    }
                }
                CK(hipMalloc(&lv.d_modup_scale, sizeof(double) * ell));
                CK(hipMemcpy(lv.d_modup_scale, sc.data(), sizeof(double) * ell, hipMemcpyHostToDevice));
            }
            CK(upload_plans(plans.data(), lv.ndig, max_src, &lv.modup));

            BConvPlan down;
            uint32_t src_ids[kMaxSrc];
            uint16_t src_limb[kMaxSrc];
            std::vector<uint32_t> dst_ids(ell);
            std::vector<uint16_t> dst_limb(ell);
            lv.special_map.n = K;
            for (uint32_t k = 0; k < K; ++k) {
                src_ids[k] = L + k;
                src_limb[k] = (uint16_t)(ell + k);
                lv.special_map.off[k] = (uint16_t)(ell + k);
                lv.special_map.mod[k] = (uint8_t)(L + k);
            }
            lv.q_map.n = ell;
            for (uint32_t i = 0; i < ell; ++i) {
                dst_ids[i] = i;
                dst_limb[i] = (uint16_t)i;
                lv.q_map.off[i] = (uint16_t)i;
                lv.q_map.mod[i] = (uint8_t)i;
            }
            fill_bconv_plan(c, &down, src_ids, src_limb, K, dst_ids.data(), dst_limb.data(), ell);
            CK(upload_plans(&down, 1, K, &lv.moddown));

            if (ell >= 2 && K + 1 <= (uint32_t)kMaxSrc) {
                BConvPlan merged;
                uint32_t m_ids[kMaxSrc];
                uint16_t m_limb[kMaxSrc];
                lv.merged_map.n = K + 1;
                for (uint32_t k = 0; k <= K; ++k) {
                    m_ids[k] = k < K ? L + k : ell - 1;
                    m_limb[k] = (uint16_t)(k < K ? ell + k : ell - 1);
                    lv.merged_map.off[k] = m_limb[k];
                    lv.merged_map.mod[k] = (uint8_t)m_ids[k];
                }
                lv.last_map.n = 1;
                lv.last_map.off[0] = (uint16_t)(ell - 1);
                lv.last_map.mod[0] = (uint8_t)(ell - 1);
                fill_bconv_plan(c, &merged, m_ids, m_limb, K + 1, dst_ids.data(), dst_limb.data(), ell - 1);
                CK(upload_plans(&merged, 1, K + 1, &lv.merged));
                std::vector<double> sc(K + 1), dinv(ell - 1);
                for (uint32_t k = 0; k <= K; ++k) {
                    const uint64_t sk = c->mod[m_ids[k]];
                    sc[k] = (double)h_mulmod((uint64_t)merged.src_inv[k], h_invmod(N % sk, sk), sk);
                }
                const uint64_t qlast = c->mod[ell - 1];
                uint64_t pl = 1;
                for (uint32_t k = 0; k < K; ++k) pl = h_mulmod(pl, c->mod[L + k] % qlast, qlast);
                lv.Pmod_last = (double)pl;
                for (uint32_t i = 0; i + 1 < ell; ++i) {
                    const uint64_t qi = c->mod[i];
                    uint64_t D = qlast % qi;
                    for (uint32_t k = 0; k < K; ++k) D = h_mulmod(D, c->mod[L + k] % qi, qi);
                    dinv[i] = (double)h_invmod(D, qi);
                }
                CK(hipMalloc(&lv.d_merged_scale, sizeof(double) * (K + 1)));
                CK(hipMemcpy(lv.d_merged_scale, sc.data(), sizeof(double) * (K + 1), hipMemcpyHostToDevice));
                CK(hipMalloc(&lv.d_Dinv, sizeof(double) * (ell - 1)));
                CK(hipMemcpy(lv.d_Dinv, dinv.data(), sizeof(double) * (ell - 1), hipMemcpyHostToDevice));
            }
            if (ell >= 2) {
                std::vector<double> ql(ell - 1);
                for (uint32_t i = 0; i + 1 < ell; ++i) ql[i] = (double)h_invmod(c->mod[ell - 1] % c->mod[i], c->mod[i]);
                CK(hipMalloc(&lv.d_qlinv, sizeof(double) * (ell - 1)));
                CK(hipMemcpy(lv.d_qlinv, ql.data(), sizeof(double) * (ell - 1), hipMemcpyHostToDevice));
            }
        }
    }
    *out = c;
    return KS_OK;
fail:
    ks_ctx_destroy(c);
    return rc;
}
