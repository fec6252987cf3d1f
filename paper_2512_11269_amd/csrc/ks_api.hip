// The extern "C" entry points: argument checks, workspace carving and the kernel chains.
#include <algorithm>

#include "ks_internal.hpp"

using namespace ks;

namespace {

// Ciphertexts processed per pass of a pipeline; bounds the workspace.  Eight fill every launch and keep more of the
// intermediates in the last-level cache than sixteen (3-4 % faster on batched key-switches and multiplications).
constexpr uint32_t kChunk = 8;
constexpr uint32_t kRotGroup = 4;  // hoisted rotations per gather launch (larger groups measured no faster); bounds the workspace

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int finish(const char* where) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e, where);
        return KS_EHIP;
    }
    return KS_OK;
}

struct KsWorkspace {  // element counts (uint64 words) for a chunk of `bc` ciphertexts
    uint64_t coeff, lifted, acc, conv;
    uint64_t accq;  // ciphertext limbs of the accumulators in packed form, [bc][2][ell][N] residues
    uint64_t total() const { return coeff + lifted + acc + conv + accq; }
};

// 64-bit words that n residues take in packed form (32-bit low words, then the bytes above; each part 8-byte aligned)
static uint64_t packed_words(uint64_t n) { return (n + 1) / 2 + (n + 7) / 8; }

// the packed tensor of n residues that starts at `words`
static PackedDigits packed_at(uint64_t* words, uint64_t n) {
    return PackedDigits{reinterpret_cast<uint32_t*>(words), reinterpret_cast<uint8_t*>(words + (n + 1) / 2)};
}

KsWorkspace ks_ws_words(const ks_ctx* c, const Level& lv, uint32_t bc) {
    const uint64_t N = c->N;
    KsWorkspace w;
    w.coeff = (uint64_t)bc * lv.ell * N;
    w.lifted = (uint64_t)bc * lv.ndig * lv.E * N;
    w.acc = (uint64_t)bc * 2 * lv.E * N;
    w.conv = (uint64_t)bc * 2 * lv.ell * N;
    w.accq = packed_words(w.conv);
    return w;
}

// Decompose and raise: d (evaluation domain, `bc` polynomials d_ps words apart) -> lifted [bc][ndig][E][N].
// The raised limbs stop after the column half of the forward transform (raw doubles); the row half is left to the
// fused inner product, or to mod_up_for_gather below.
void mod_up(const ks_ctx* c, const Level& lv, const void* d, uint64_t d_ps, uint64_t* coeff, uint64_t* lifted, uint32_t bc,
            hipStream_t s, bool d_words32 = false) {
    const uint64_t N = c->N, coeff_ps = (uint64_t)lv.ell * N, lifted_ps = (uint64_t)lv.ndig * lv.E * N;
    launch_ntt_inv_rows(c, lv.q_map, XformIO{d, coeff, d_ps, coeff_ps, bc}, s, d_words32);
    // the column half also multiplies by N^-1 (D_j/q_i)^-1 and leaves canonical doubles for the conversion
    launch_ntt_inv_cols(c, lv.q_map, coeff, coeff_ps, bc, lv.d_modup_scale, true, true, s);
    // algorithmic fp64 work per coefficient: 3 FMAs per source x target plus the 6-addition split of the source shared
    // by four targets (4.5 in all), then per target one reduction and the column stages (8 per butterfly, half a
    // butterfly per point and stage)
    double ops = 0.0;
    for (uint32_t j = 0; j < lv.ndig; ++j) {
        const double a = lv.digit_hi[j] - lv.digit_lo[j];
        ops += a * (lv.E - a) * 4.5;
    }
    ops += lv.n_new * (3.0 + 4.0 * (c->logN - 8));
    launch_bconv_ntt_cols(c, lv.modup, lv.ell + lv.n_new, coeff, coeff_ps, lifted, lifted_ps, bc, s, ops);
}

// Words of workspace the gathers' sources of a chunk take: the finished raised digits as 32-bit words (words32), or as
// 32-bit low words plus high bytes, own limbs included (64-bit operands).
static uint64_t gather_words(const KsWorkspace& w, bool words32) { return (w.lifted + 1) / 2 + (words32 ? 0 : (w.lifted + 7) / 8); }

// mod_up finished for the rotation gathers: `region` (gather_words() words) ends as the bundle the gathers read, the
// raised digits as canonical evaluation-domain residues and d's own limbs in their digits' slots, 32-bit words (words32)
// or packed.  `lifted` is only scratch here.
static GatherSources mod_up_for_gather(const ks_ctx* c, const Level& lv, const void* d, uint64_t d_ps, uint64_t* coeff,
                                       uint64_t* lifted, uint64_t* region, uint32_t bc, hipStream_t s, bool words32) {
    mod_up(c, lv, d, d_ps, coeff, lifted, bc, s, words32);
    const uint64_t lifted_words = (uint64_t)bc * lv.ndig * lv.E * c->N;
    const PackedDigits bundle{reinterpret_cast<uint32_t*>(region),
                              words32 ? nullptr : reinterpret_cast<uint8_t*>(region + (lifted_words + 1) / 2)};
    launch_gather_bundle_rows(c, lv, lifted, d, d_ps, words32, bundle, bc, s);
    return GatherSources{bundle.lo, bundle.hi};
}

// algorithmic fp64 work per coefficient of the ModDown conversion + column half (see mod_up)
static double moddown_ops(const ks_ctx* c, const Level& lv) {
    return (double)c->K * lv.ell * 4.5 + lv.ell * (3.0 + 4.0 * (c->logN - 8));
}

// Division by P of both accumulators, optional addend: INTT of the special limbs (in place), fused base
// conversion + column half, fused row half + (acc - conv) P^-1.
// accq: the ciphertext limbs of the accumulators are there, packed, instead of in acc.
// addend_packed (with accq): the addend is there, [b][2][ell][N] packed (addend_bs in elements), instead of at addend.
void mod_down(const ks_ctx* c, const Level& lv, uint64_t* acc, uint64_t* conv, void* out, uint64_t out_bs,
              const uint64_t* addend, uint64_t addend_bs, uint32_t addend_comps, uint32_t galois, uint32_t bc,
              bool special_rows_done, hipStream_t s, bool out_words32 = false, const PackedDigits* accq = nullptr,
              const PackedDigits* addend_packed = nullptr) {
    const uint64_t N = c->N, acc_ps = (uint64_t)lv.E * N, conv_ps = (uint64_t)lv.ell * N;
    // the fused inner product already ran the row half of the inverse transform on the special limbs
    if (!special_rows_done) launch_ntt_inv_rows(c, lv.special_map, XformIO{acc, acc, acc_ps, acc_ps, 2 * bc}, s);
    launch_ntt_inv_cols(c, lv.special_map, acc, acc_ps, 2 * bc, c->d_moddown_scale, true, true, s);
    launch_bconv_ntt_cols(c, lv.moddown, c->K + lv.ell, acc, acc_ps, conv, conv_ps, 2 * bc, s, moddown_ops(c, lv));
    launch_rows_moddown_finish(c, lv, acc, conv, out, out_bs, addend, addend_bs, addend_comps, galois, bc, s, nullptr, out_words32, accq,
                               addend_packed);
}

}  // namespace

extern "C" size_t ks_workspace_bytes(const ks_ctx* c, int op, uint32_t ell, uint32_t batch, uint32_t n_rot) {
    if (!c || c->K == 0 || ell < 1 || ell > c->L || batch == 0) return 0;
    const Level& lv = c->levels[ell - 1];
    const uint32_t bc = std::min(batch, kChunk);
    const uint64_t N = c->N;
    uint64_t words = ks_ws_words(c, lv, bc).total();
    switch (op) {
        case KS_OP_KEYSWITCH: break;
        case KS_OP_ROTATE_HOISTED:
        case KS_OP_ROTATE_HOISTED_U32:
            if (n_rot == 0) return 0;
            // accumulators and converted limbs for a whole group of rotations
            words += (uint64_t)(std::min(n_rot, kRotGroup) - 1) * bc * (2 * lv.E + 2 * ell) * N;
            // the gathers' sources; the ciphertext limbs of a group's accumulators, packed
            words += gather_words(ks_ws_words(c, lv, bc), op == KS_OP_ROTATE_HOISTED_U32);
            words += (uint64_t)(std::min(n_rot, kRotGroup) - 1) * ks_ws_words(c, lv, bc).accq;
            break;
        case KS_OP_BSGS:
        case KS_OP_BSGS_U32: {
            // accumulators of the outer level, inner result [bc][2][ell], the gathers' sources of both levels (the
            // inner results are 64-bit words either way)
            const KsWorkspace w = ks_ws_words(c, lv, bc);
            words += w.acc + (uint64_t)bc * 2 * ell * N + gather_words(w, op == KS_OP_BSGS_U32) + gather_words(w, false);
            break;
        }
        case KS_OP_HMULT_RELIN_RESCALE:
            if (ell < 2) return 0;
            // d2 [bc][ell], (d0, d1) packed like the accumulator limbs, sum [bc][2][ell], last limb [2 bc], spread [2 bc][ell-1]
            words += (uint64_t)bc * (ell + 2 * ell + 2 + 2 * (ell - 1)) * N + ks_ws_words(c, lv, bc).accq;
            break;
        default: return 0;
    }
    return (size_t)words * sizeof(uint64_t);
}

static int check_map_args(const ks_ctx* c, const void* data, const uint32_t* mod_ids, uint32_t nlimbs, LimbMap* map) {
    if (!c || !data || !mod_ids || nlimbs == 0 || nlimbs > (uint32_t)kMaxLimbs || !aligned16(data)) return KS_EINVAL;
    map->n = nlimbs;
    for (uint32_t i = 0; i < nlimbs; ++i) {
        if (mod_ids[i] >= c->M) return KS_EINVAL;
        map->off[i] = (uint16_t)i;
        map->mod[i] = (uint8_t)mod_ids[i];
    }
    return KS_OK;
}

extern "C" int ntt_fwd(const ks_ctx* c, uint64_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream) {
    LimbMap map;
    int rc = check_map_args(c, data, mod_ids, nlimbs, &map);
    if (rc != KS_OK) return rc;
    if (batch == 0) return KS_OK;
    if ((uint64_t)batch * nlimbs > (1u << 26)) return KS_EINVAL;
    const uint64_t ps = (uint64_t)nlimbs * c->N;
    launch_ntt_fwd(c, map, XformIO{data, data, ps, ps, batch}, static_cast<hipStream_t>(stream));
    return finish("ntt_fwd");
}

extern "C" int ntt_inv(const ks_ctx* c, uint64_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream) {
    LimbMap map;
    int rc = check_map_args(c, data, mod_ids, nlimbs, &map);
    if (rc != KS_OK) return rc;
    if (batch == 0) return KS_OK;
    if ((uint64_t)batch * nlimbs > (1u << 26)) return KS_EINVAL;
    const uint64_t ps = (uint64_t)nlimbs * c->N;
    launch_ntt_inv(c, map, XformIO{data, data, ps, ps, batch}, static_cast<hipStream_t>(stream));
    return finish("ntt_inv");
}

static bool moduli_fit_u32(const ks_ctx* c) {
    for (uint64_t m : c->mod)
        if (m >> 32) return false;
    return true;
}

static int ntt_u32(const ks_ctx* c, uint32_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream,
                   bool inverse) {
    LimbMap map;
    int rc = check_map_args(c, data, mod_ids, nlimbs, &map);
    if (rc != KS_OK) return rc;
    if (!moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if ((uint64_t)batch * nlimbs > (1u << 26)) return KS_EINVAL;
    launch_ntt_u32(c, map, data, (uint64_t)nlimbs * c->N, batch, inverse, static_cast<hipStream_t>(stream));
    return finish(inverse ? "ntt_inv_u32" : "ntt_fwd_u32");
}

extern "C" int ntt_fwd_u32(const ks_ctx* c, uint32_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream) {
    return ntt_u32(c, data, mod_ids, nlimbs, batch, stream, false);
}

extern "C" int ntt_inv_u32(const ks_ctx* c, uint32_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream) {
    return ntt_u32(c, data, mod_ids, nlimbs, batch, stream, true);
}

// Key of a registered conversion: n_src, source ids, target ids.  Returns KS_OK or KS_EINVAL.
static int bconv_key(const ks_ctx* c, const uint32_t* src_ids, uint32_t n_src, const uint32_t* dst_ids, uint32_t n_dst,
                     std::vector<uint32_t>* key) {
    if (!c || !src_ids || !dst_ids) return KS_EINVAL;
    if (n_src == 0 || n_src > (uint32_t)kMaxSrc || n_dst == 0 || n_dst > 255) return KS_EINVAL;
    key->push_back(n_src);
    for (uint32_t i = 0; i < n_src; ++i) {
        if (src_ids[i] >= c->M) return KS_EINVAL;
        for (uint32_t k = 0; k < i; ++k)
            if (src_ids[k] == src_ids[i]) return KS_EINVAL;
        key->push_back(src_ids[i]);
    }
    for (uint32_t t = 0; t < n_dst; ++t) {
        if (dst_ids[t] >= c->M) return KS_EINVAL;
        key->push_back(dst_ids[t]);
    }
    return KS_OK;
}

extern "C" int bconv_prepare(ks_ctx* c, const uint32_t* src_ids, uint32_t n_src, const uint32_t* dst_ids, uint32_t n_dst) {
    std::vector<uint32_t> key;
    int rc = bconv_key(c, src_ids, n_src, dst_ids, n_dst, &key);
    if (rc != KS_OK) return rc;
    std::lock_guard<std::mutex> lock(c->mu);
    if (c->bconv_cache.count(key)) return KS_OK;
    if (hipSetDevice(c->device) != hipSuccess) return KS_EHIP;
    std::vector<BConvPlan> plan(1);
    uint16_t src_limb[kMaxSrc];
    std::vector<uint16_t> dst_limb(n_dst);
    for (uint32_t i = 0; i < n_src; ++i) src_limb[i] = (uint16_t)i;
    for (uint32_t t = 0; t < n_dst; ++t) dst_limb[t] = (uint16_t)t;
    fill_bconv_plan(c, plan.data(), src_ids, src_limb, n_src, dst_ids, dst_limb.data(), n_dst);
    PlanSet set;
    hipError_t e = upload_plans(plan.data(), 1, n_src, &set);
    if (e != hipSuccess) {
        set_hip_error(e, "bconv_prepare: table upload");
        return KS_EHIP;
    }
    c->bconv_cache[key] = set;
    return KS_OK;
}

static int bconv_impl(const ks_ctx* c, const void* in, const uint32_t* src_ids, uint32_t n_src, void* out, const uint32_t* dst_ids,
                      uint32_t n_dst, uint32_t batch, void* stream, bool words32) {
    if (!in || !out || !aligned16(in) || !aligned16(out)) return KS_EINVAL;
    std::vector<uint32_t> key;
    int rc = bconv_key(c, src_ids, n_src, dst_ids, n_dst, &key);
    if (rc != KS_OK) return rc;
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    PlanSet set;
    {
        std::lock_guard<std::mutex> lock(c->mu);
        auto it = c->bconv_cache.find(key);
        if (it == c->bconv_cache.end()) return KS_ENOTPREPARED;  // compute calls never allocate: register with bconv_prepare
        set = it->second;
    }
    if (batch == 0) return KS_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, word = words32 ? 4 : 8;
    for (uint32_t b0 = 0; b0 < batch; b0 += 32768) {
        const uint32_t nb = std::min(batch - b0, 32768u);
        const char* ip = static_cast<const char*>(in) + (uint64_t)b0 * n_src * N * word;
        char* op = static_cast<char*>(out) + (uint64_t)b0 * n_dst * N * word;
        // Which kernel (KS_OPT_BCONV_KERNEL overrides): launches of a few polynomials run about twice as fast on the
        // matrix-core kernel (twice the workgroups, targets walked six at a time: 10.9 against 20.9 us for one polynomial,
        // 8 -> 24 moduli at N = 2^16); once the chip is full both are bandwidth-bound and the vector kernel is 9-12 %
        // ahead.  32-bit words always take the vector kernel.
        const bool few = (uint64_t)nb * (N / 256) < 1024;
        const int kernel = c->opt[KS_OPT_BCONV_KERNEL] ? c->opt[KS_OPT_BCONV_KERNEL] : (few ? 2 : 1);
        if (!words32 && kernel == 2)
            launch_bconv_mfma(c, set, n_src + n_dst, reinterpret_cast<const uint64_t*>(ip), (uint64_t)n_src * N,
                              reinterpret_cast<uint64_t*>(op), (uint64_t)n_dst * N, nb, s);
        else
            launch_bconv(c, set, n_src + n_dst, ip, (uint64_t)n_src * N, op, (uint64_t)n_dst * N, nb, s, words32);
    }
    return finish(words32 ? "bconv_u32" : "bconv");
}

extern "C" int bconv(const ks_ctx* c, const uint64_t* in, const uint32_t* src_ids, uint32_t n_src, uint64_t* out,
                     const uint32_t* dst_ids, uint32_t n_dst, uint32_t batch, void* stream) {
    return bconv_impl(c, in, src_ids, n_src, out, dst_ids, n_dst, batch, stream, false);
}

extern "C" int bconv_u32(const ks_ctx* c, const uint32_t* in, const uint32_t* src_ids, uint32_t n_src, uint32_t* out,
                         const uint32_t* dst_ids, uint32_t n_dst, uint32_t batch, void* stream) {
    return bconv_impl(c, in, src_ids, n_src, out, dst_ids, n_dst, batch, stream, true);
}

static int check_pipeline_args(const ks_ctx* c, uint32_t ell, uint32_t min_ell, const void* a, const void* b, const void* o,
                               const void* ws) {
    if (!c || c->K == 0 || !a || !b || !o || !aligned16(a) || !aligned16(b) || !aligned16(o)) return KS_EINVAL;
    if (ell < min_ell || ell > c->L) return KS_EINVAL;
    if (!ws || !aligned16(ws)) return KS_EWORKSPACE;
    return KS_OK;
}

// d, evk and out in 64-bit words, or all three in 32-bit words (words32; every modulus then below 2^32).
int ks::keyswitch_impl(const ks_ctx* c, const void* d, uint32_t ell, const void* evk, void* out, uint32_t batch, void* ws,
                          size_t ws_bytes, void* stream, bool words32) {
    int rc = check_pipeline_args(c, ell, 1, d, evk, out, ws);
    if (rc != KS_OK) return rc;
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if (ws_bytes < ks_workspace_bytes(c, KS_OP_KEYSWITCH, ell, batch, 0)) return KS_EWORKSPACE;
    const Level& lv = c->levels[ell - 1];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, d_ps = (uint64_t)ell * N, out_bs = 2ull * ell * N, word = words32 ? 4 : 8;
    for (uint32_t b0 = 0; b0 < batch; b0 += kChunk) {
        const uint32_t bc = std::min(batch - b0, kChunk);
        const KsWorkspace w = ks_ws_words(c, lv, bc);
        uint64_t* coeff = static_cast<uint64_t*>(ws);
        uint64_t* lifted = coeff + w.coeff;
        uint64_t* acc = lifted + w.lifted;
        uint64_t* conv = acc + w.acc;
        const PackedDigits accq = packed_at(conv + w.conv, w.conv);
        const char* dc = static_cast<const char*>(d) + (uint64_t)b0 * d_ps * word;
        mod_up(c, lv, dc, d_ps, coeff, lifted, bc, s, words32);
        launch_rows_inner_product(c, lv, dc, d_ps, lifted, evk, acc, bc, s, words32, words32, &accq, ell);
        mod_down(c, lv, acc, conv, static_cast<char*>(out) + (uint64_t)b0 * out_bs * word, out_bs, nullptr, 0, 0, 1, bc, true, s, words32,
                 &accq);
    }
    return finish(words32 ? "ks_keyswitch_u32" : "ks_keyswitch");
}

extern "C" int ks_keyswitch(const ks_ctx* c, const uint64_t* d, uint32_t ell, const uint64_t* evk, uint64_t* out, uint32_t batch,
                            void* ws, size_t ws_bytes, void* stream) {
    return keyswitch_impl(c, d, ell, evk, out, batch, ws, ws_bytes, stream, false);
}

extern "C" int ks_keyswitch_u32(const ks_ctx* c, const uint32_t* d, uint32_t ell, const uint32_t* evk, uint32_t* out, uint32_t batch,
                                void* ws, size_t ws_bytes, void* stream) {
    return keyswitch_impl(c, d, ell, evk, out, batch, ws, ws_bytes, stream, true);
}

// ct, keys and out in 64-bit words, or all in 32-bit words (words32).
static int rotate_hoisted_impl(const ks_ctx* c, const void* ct, uint32_t ell, const uint32_t* galois, const void* const* rot_keys,
                               uint32_t n_rot, void* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream, bool words32) {
    int rc = check_pipeline_args(c, ell, 1, ct, ct, out, ws);
    if (rc != KS_OK) return rc;
    if (!galois || !rot_keys || n_rot == 0) return KS_EINVAL;
    for (uint32_t r = 0; r < n_rot; ++r) {
        if ((galois[r] & 1u) == 0 || galois[r] >= 2u * c->N) return KS_EINVAL;
        if (!rot_keys[r] || !aligned16(rot_keys[r])) return KS_EINVAL;
    }
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if (ws_bytes < ks_workspace_bytes(c, words32 ? KS_OP_ROTATE_HOISTED_U32 : KS_OP_ROTATE_HOISTED, ell, batch, n_rot))
        return KS_EWORKSPACE;
    const Level& lv = c->levels[ell - 1];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, ct_bs = 2ull * ell * N, out_bs = (uint64_t)n_rot * 2 * ell * N, word = words32 ? 4 : 8;
    for (uint32_t b0 = 0; b0 < batch; b0 += kChunk) {
        const uint32_t bc = std::min(batch - b0, kChunk);
        const KsWorkspace w = ks_ws_words(c, lv, bc);
        // The gathers read c1 and its finished raised digits in a compact form (32-bit words, or 32-bit low words plus
        // high bytes for 64-bit operands: their traffic bounds the gather kernels); the last kernel's addend c0 is gathered
        // from the ciphertext in its own word size.
        uint64_t* region = static_cast<uint64_t*>(ws);
        uint64_t* coeff = region + gather_words(w, words32);
        const char* c0 = static_cast<const char*>(ct) + (uint64_t)b0 * ct_bs * word;
        const void* c1 = c0 + (uint64_t)ell * N * word;
        uint64_t* lifted = coeff + w.coeff;
        uint64_t* acc = lifted + w.lifted;
        // finished once, shared by every rotation
        const GatherSources digits = mod_up_for_gather(c, lv, c1, ct_bs, coeff, lifted, region, bc, s, words32);
        // Rotations go in groups: one gather launch forms the accumulators of the whole group (the raised digits then come
        // from memory once per group), the inverse transform and the conversion run over the group as one batch, and only
        // the last kernel, which adds sigma_g(c0) through a rotation's own permutation, runs per rotation.
        const uint32_t group = std::min(n_rot, kRotGroup);
        uint64_t* conv = acc + (uint64_t)group * w.acc;
        // ciphertext limbs of the group's accumulators, packed: [group][bc][2][ell][N]
        const uint64_t accq_n = w.conv;
        const PackedDigits accq = packed_at(conv + (uint64_t)group * w.conv, (uint64_t)group * accq_n);
        const uint64_t acc_ps = (uint64_t)lv.E * N, conv_ps = (uint64_t)ell * N;
        for (uint32_t r0 = 0; r0 < n_rot; r0 += group) {
            MacRotations rot;
            rot.n = std::min(n_rot - r0, group);
            for (uint32_t r = 0; r < rot.n; ++r) {
                rot.galois[r] = galois[r0 + r];
                rot.key[r] = rot_keys[r0 + r];
                rot.pt[r] = nullptr;
            }
            launch_inner_product(c, lv, digits, rot, acc, accq, bc, s, words32);
            const uint32_t polys = 2 * rot.n * bc;
            launch_ntt_inv_rows(c, lv.special_map, XformIO{acc, acc, acc_ps, acc_ps, polys}, s);
            launch_ntt_inv_cols(c, lv.special_map, acc, acc_ps, polys, c->d_moddown_scale, true, true, s);
            launch_bconv_ntt_cols(c, lv.moddown, c->K + lv.ell, acc, acc_ps, conv, conv_ps, polys, s, moddown_ops(c, lv));
            for (uint32_t r = 0; r < rot.n; ++r) {
                const PackedDigits accq_r{accq.lo + (uint64_t)r * accq_n, accq.hi + (uint64_t)r * accq_n};
                launch_rows_moddown_finish(c, lv, nullptr, conv + (uint64_t)r * w.conv,
                                           static_cast<char*>(out) + ((uint64_t)b0 * out_bs + (uint64_t)(r0 + r) * 2 * ell * N) * word,
                                           out_bs, c0, ct_bs, 1, galois[r0 + r], bc, s, nullptr, words32, &accq_r, nullptr, words32);
            }
        }
    }
    return finish(words32 ? "ks_rotate_hoisted_u32" : "ks_rotate_hoisted");
}

extern "C" int ks_rotate_hoisted(const ks_ctx* c, const uint64_t* ct, uint32_t ell, const uint32_t* galois,
                                 const uint64_t* const* rot_keys, uint32_t n_rot, uint64_t* out, uint32_t batch, void* ws,
                                 size_t ws_bytes, void* stream) {
    return rotate_hoisted_impl(c, ct, ell, galois, reinterpret_cast<const void* const*>(rot_keys), n_rot, out, batch, ws, ws_bytes,
                               stream, false);
}

extern "C" int ks_rotate_hoisted_u32(const ks_ctx* c, const uint32_t* ct, uint32_t ell, const uint32_t* galois,
                                     const uint32_t* const* rot_keys, uint32_t n_rot, uint32_t* out, uint32_t batch, void* ws,
                                     size_t ws_bytes, void* stream) {
    return rotate_hoisted_impl(c, ct, ell, galois, reinterpret_cast<const void* const*>(rot_keys), n_rot, out, batch, ws, ws_bytes,
                               stream, true);
}

// Galois elements, keys and plaintexts of a rotate-multiply-accumulate: g = 1 needs no key, a null plaintext is 1.
static int check_mac_rotations(const ks_ctx* c, const uint32_t* galois, const void* const* keys, const void* const* pts,
                               uint32_t n) {
    if (!galois || !keys || n == 0) return KS_EINVAL;
    for (uint32_t r = 0; r < n; ++r) {
        if ((galois[r] & 1u) == 0 || galois[r] >= 2u * c->N) return KS_EINVAL;
        if (galois[r] != 1 && (!keys[r] || !aligned16(keys[r]))) return KS_EINVAL;
        if (pts && pts[r] && !aligned16(pts[r])) return KS_EINVAL;
    }
    return KS_OK;
}

// u (+)= sum_r pt_r * rot_{g_r}(ct) for all n rotations, in launches of kMacRotations
static void rotate_mac_all(const ks_ctx* c, const Level& lv, const void* ct, uint64_t ct_bs, const GatherSources& src,
                           const uint32_t* galois, const void* const* keys, const void* const* pts, uint32_t n, uint64_t* u,
                           uint32_t bc, bool accumulate, hipStream_t s, bool key_words32 = false) {
    for (uint32_t r0 = 0; r0 < n; r0 += kMacRotations) {
        MacRotations rot;
        rot.n = std::min<uint32_t>(n - r0, kMacRotations);
        for (uint32_t r = 0; r < rot.n; ++r) {
            rot.galois[r] = galois[r0 + r];
            rot.key[r] = keys[r0 + r];
            rot.pt[r] = pts ? pts[r0 + r] : nullptr;
        }
        launch_rotate_mac(c, lv, ct, ct_bs, src, rot, u, bc, accumulate || r0 != 0, s, key_words32);
    }
}

static int rotate_mac_impl(const ks_ctx* c, const void* ct, uint32_t ell, const uint32_t* galois, const void* const* rot_keys,
                           const void* const* pts, uint32_t n_rot, void* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream,
                           bool words32) {
    int rc = check_pipeline_args(c, ell, 1, ct, ct, out, ws);
    if (rc != KS_OK) return rc;
    if (!pts || (rc = check_mac_rotations(c, galois, rot_keys, pts, n_rot)) != KS_OK) return KS_EINVAL;
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if (ws_bytes < ks_workspace_bytes(c, words32 ? KS_OP_ROTATE_HOISTED_U32 : KS_OP_ROTATE_HOISTED, ell, batch, n_rot))
        return KS_EWORKSPACE;
    const Level& lv = c->levels[ell - 1];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, ct_bs = 2ull * ell * N, word = words32 ? 4 : 8;
    for (uint32_t b0 = 0; b0 < batch; b0 += kChunk) {
        const uint32_t bc = std::min(batch - b0, kChunk);
        const KsWorkspace w = ks_ws_words(c, lv, bc);
        // the gathers read c1 and its finished raised digits in a compact form (see rotate_hoisted_impl)
        const char* c0 = static_cast<const char*>(ct) + (uint64_t)b0 * ct_bs * word;
        uint64_t* region = static_cast<uint64_t*>(ws);
        uint64_t* coeff = region + gather_words(w, words32);
        uint64_t* lifted = coeff + w.coeff;
        uint64_t* acc = lifted + w.lifted;
        uint64_t* conv = acc + w.acc;
        // finished once, shared by every rotation
        const GatherSources digits = mod_up_for_gather(c, lv, c0 + (uint64_t)ell * N * word, ct_bs, coeff, lifted, region, bc, s, words32);
        rotate_mac_all(c, lv, c0, ct_bs, digits, galois, rot_keys, pts, n_rot, acc, bc, false, s, words32);
        mod_down(c, lv, acc, conv, static_cast<char*>(out) + (uint64_t)b0 * ct_bs * word, ct_bs, nullptr, 0, 0, 1, bc, false, s, words32);
    }
    return finish(words32 ? "ks_rotate_mac_hoisted_u32" : "ks_rotate_mac_hoisted");
}

extern "C" int ks_rotate_mac_hoisted(const ks_ctx* c, const uint64_t* ct, uint32_t ell, const uint32_t* galois,
                                     const uint64_t* const* rot_keys, const uint64_t* const* pts, uint32_t n_rot, uint64_t* out,
                                     uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return rotate_mac_impl(c, ct, ell, galois, reinterpret_cast<const void* const*>(rot_keys),
                           reinterpret_cast<const void* const*>(pts), n_rot, out, batch, ws, ws_bytes, stream, false);
}

extern "C" int ks_rotate_mac_hoisted_u32(const ks_ctx* c, const uint32_t* ct, uint32_t ell, const uint32_t* galois,
                                         const uint32_t* const* rot_keys, const uint32_t* const* pts, uint32_t n_rot, uint32_t* out,
                                         uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return rotate_mac_impl(c, ct, ell, galois, reinterpret_cast<const void* const*>(rot_keys),
                           reinterpret_cast<const void* const*>(pts), n_rot, out, batch, ws, ws_bytes, stream, true);
}

// ct, keys, plaintexts and out in 64-bit words, or all in 32-bit words (words32).
static int bsgs_impl(const ks_ctx* c, const void* ct, uint32_t ell, const uint32_t* baby_galois, const void* const* bkeys, uint32_t n1,
                     const uint32_t* giant_galois, const void* const* gkeys, uint32_t n2, const void* const* ptv, void* out,
                     uint32_t batch, void* ws, size_t ws_bytes, void* stream, bool words32) {
    int rc = check_pipeline_args(c, ell, 1, ct, ct, out, ws);
    if (rc != KS_OK) return rc;
    if (!ptv || check_mac_rotations(c, giant_galois, gkeys, nullptr, n2) != KS_OK) return KS_EINVAL;
    for (uint32_t g = 0; g < n2; ++g)
        if (check_mac_rotations(c, baby_galois, bkeys, ptv + (size_t)g * n1, n1) != KS_OK) return KS_EINVAL;
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if (ws_bytes < ks_workspace_bytes(c, words32 ? KS_OP_BSGS_U32 : KS_OP_BSGS, ell, batch, 0)) return KS_EWORKSPACE;
    const Level& lv = c->levels[ell - 1];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, ct_bs = 2ull * ell * N, word = words32 ? 4 : 8;
    for (uint32_t b0 = 0; b0 < batch; b0 += kChunk) {
        const uint32_t bc = std::min(batch - b0, kChunk);
        const KsWorkspace w = ks_ws_words(c, lv, bc);
        // The gathers of the inner level read the input ciphertext and its finished raised digits in a compact form (see
        // rotate_hoisted_impl); the inner results are 64-bit words either way, so the outer level reads the packed form.
        const char* c0 = static_cast<const char*>(ct) + (uint64_t)b0 * ct_bs * word;
        uint64_t* region = static_cast<uint64_t*>(ws);   // sources of the inner level, shared by every baby step of every giant step
        uint64_t* region_v = region + gather_words(w, words32);   // sources of the outer level: the current inner result
        uint64_t* coeff = region_v + gather_words(w, false);
        uint64_t* lifted = coeff + w.coeff;          // scratch of a ModUp
        uint64_t* acc = lifted + w.lifted;           // inner sum of the current giant step
        uint64_t* conv = acc + w.acc;
        uint64_t* acc_outer = conv + w.conv;         // outer sum over the giant steps
        uint64_t* v = acc_outer + w.acc;             // [bc][2][ell][N] inner result of the current giant step (64-bit words)
        const GatherSources digits = mod_up_for_gather(c, lv, c0 + (uint64_t)ell * N * word, ct_bs, coeff, lifted, region, bc, s, words32);
        GatherSources digits_v{};
        for (uint32_t g = 0; g < n2; ++g) {
            rotate_mac_all(c, lv, c0, ct_bs, digits, baby_galois, bkeys, ptv + (size_t)g * n1, n1, acc, bc, false, s, words32);
            mod_down(c, lv, acc, conv, v, ct_bs, nullptr, 0, 0, 1, bc, false, s);
            if (giant_galois[g] != 1) digits_v = mod_up_for_gather(c, lv, v + (uint64_t)ell * N, ct_bs, coeff, lifted, region_v, bc, s, false);
            // Galois element 1 gathers nothing; the packed form still says that v holds 64-bit words
            else digits_v = GatherSources{reinterpret_cast<const uint32_t*>(region_v), reinterpret_cast<const uint8_t*>(region_v)};
            rotate_mac_all(c, lv, v, ct_bs, digits_v, giant_galois + g, gkeys + g, nullptr, 1, acc_outer, bc, g != 0, s, words32);
        }
        mod_down(c, lv, acc_outer, conv, static_cast<char*>(out) + (uint64_t)b0 * ct_bs * word, ct_bs, nullptr, 0, 0, 1, bc, false, s,
                 words32);
    }
    return finish(words32 ? "ks_bsgs_linear_transform_u32" : "ks_bsgs_linear_transform");
}

extern "C" int ks_bsgs_linear_transform(const ks_ctx* c, const uint64_t* ct, uint32_t ell, const uint32_t* baby_galois,
                                        const uint64_t* const* baby_keys, uint32_t n1, const uint32_t* giant_galois,
                                        const uint64_t* const* giant_keys, uint32_t n2, const uint64_t* const* pts, uint64_t* out,
                                        uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return bsgs_impl(c, ct, ell, baby_galois, reinterpret_cast<const void* const*>(baby_keys), n1, giant_galois,
                     reinterpret_cast<const void* const*>(giant_keys), n2, reinterpret_cast<const void* const*>(pts), out, batch, ws,
                     ws_bytes, stream, false);
}

extern "C" int ks_bsgs_linear_transform_u32(const ks_ctx* c, const uint32_t* ct, uint32_t ell, const uint32_t* baby_galois,
                                            const uint32_t* const* baby_keys, uint32_t n1, const uint32_t* giant_galois,
                                            const uint32_t* const* giant_keys, uint32_t n2, const uint32_t* const* pts, uint32_t* out,
                                            uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return bsgs_impl(c, ct, ell, baby_galois, reinterpret_cast<const void* const*>(baby_keys), n1, giant_galois,
                     reinterpret_cast<const void* const*>(giant_keys), n2, reinterpret_cast<const void* const*>(pts), out, batch, ws,
                     ws_bytes, stream, true);
}

// Division by P q_{ell-1} of acc + P addend in one conversion (ModDown merged with the rescale that would follow):
// limb ell-1 joins the special limbs as a source, the targets are q_0..q_{ell-2}.  The fused inner product has already
// run the row half of the inverse transform on the special limbs.
// accq: the ciphertext limbs below ell-1 of the accumulators, packed (limb ell-1 is a conversion source and stays in acc).
// addend: [b][2][ell][N] packed.
static void mod_down_merged(const ks_ctx* c, const Level& lv, uint64_t* acc, uint64_t* conv, void* out, uint64_t out_bs,
                            const PackedDigits& addend, uint32_t bc, hipStream_t s, bool out_words32, const PackedDigits* accq) {
    const uint64_t N = c->N, acc_ps = (uint64_t)lv.E * N, conv_ps = (uint64_t)lv.ell * N;
    launch_add_scaled_limb(c, acc, acc_ps, addend, lv.ell, lv.ell - 1, lv.Pmod_last, bc, s);
    launch_ntt_inv_rows(c, lv.last_map, XformIO{acc, acc, acc_ps, acc_ps, 2 * bc}, s);
    launch_ntt_inv_cols(c, lv.merged_map, acc, acc_ps, 2 * bc, lv.d_merged_scale, true, true, s);
    const uint32_t n_src = c->K + 1, n_dst = lv.ell - 1;
    const double ops = (double)n_src * n_dst * 4.5 + n_dst * (3.0 + 4.0 * (c->logN - 8));
    launch_bconv_ntt_cols(c, lv.merged, n_src + n_dst, acc, acc_ps, conv, conv_ps, 2 * bc, s, ops);
    const FinishScale fs{lv.d_Dinv, lv.d_qlinv, n_dst};
    launch_rows_moddown_finish(c, lv, acc, conv, out, out_bs, nullptr, 2ull * lv.ell * N, 2, 1, bc, s, &fs, out_words32, accq, &addend);
}

// cta, ctb, rlk and out in 64-bit words, or all four in 32-bit words (words32); the tensor product and everything after it
// in the workspace stay 64-bit.
static int hmult_impl(const ks_ctx* c, const void* cta, const void* ctb, uint32_t ell, const void* rlk, void* out, uint32_t batch,
                      void* ws, size_t ws_bytes, void* stream, bool merged, bool words32) {
    int rc = check_pipeline_args(c, ell, 2, cta, ctb, out, ws);
    if (rc != KS_OK) return rc;
    if (!rlk || !aligned16(rlk)) return KS_EINVAL;
    if (words32 && !moduli_fit_u32(c)) return KS_EINVAL;
    if (batch == 0) return KS_OK;
    if (ws_bytes < ks_workspace_bytes(c, KS_OP_HMULT_RELIN_RESCALE, ell, batch, 0)) return KS_EWORKSPACE;
    const Level& lv = c->levels[ell - 1];
    if (merged && !lv.merged.d_plans) return KS_EINVAL;  // K + 1 sources exceed what one conversion takes
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t N = c->N, ct_bs = 2ull * ell * N, out_bs = 2ull * (ell - 1) * N, word = words32 ? 4 : 8;
    LimbMap one;
    one.n = 1;
    one.off[0] = 0;
    one.mod[0] = (uint8_t)(ell - 1);
    for (uint32_t b0 = 0; b0 < batch; b0 += kChunk) {
        const uint32_t bc = std::min(batch - b0, kChunk);
        const KsWorkspace w = ks_ws_words(c, lv, bc);
        uint64_t* coeff = static_cast<uint64_t*>(ws);
        uint64_t* lifted = coeff + w.coeff;
        uint64_t* acc = lifted + w.lifted;
        uint64_t* conv = acc + w.acc;
        const PackedDigits accq = packed_at(conv + w.conv, w.conv);
        uint64_t* d2 = conv + w.conv + w.accq;                  // [bc][ell][N], the polynomial that is key-switched
        const uint64_t d2_ps = (uint64_t)ell * N;
        const PackedDigits dq = packed_at(d2 + (uint64_t)bc * d2_ps, w.conv);   // (d0, d1): [bc][2][ell][N] packed
        uint64_t* sum = d2 + (uint64_t)bc * d2_ps + w.accq;     // [bc][2][ell][N]
        uint64_t* last = sum + (uint64_t)bc * ct_bs;            // [2 bc][N]
        uint64_t* spread = last + (uint64_t)bc * 2 * N;         // [2 bc][ell-1][N]
        char* oc = static_cast<char*>(out) + (uint64_t)b0 * out_bs * word;
        launch_tensor_product(c, static_cast<const char*>(cta) + (uint64_t)b0 * ct_bs * word,
                              static_cast<const char*>(ctb) + (uint64_t)b0 * ct_bs * word, d2, dq, ell, bc, s, words32);
        mod_up(c, lv, d2, d2_ps, coeff, lifted, bc, s);
        launch_rows_inner_product(c, lv, d2, d2_ps, lifted, rlk, acc, bc, s, false, words32, &accq, merged ? ell - 1 : ell);
        if (merged) {
            mod_down_merged(c, lv, acc, conv, oc, out_bs, dq, bc, s, words32, &accq);
            continue;
        }
        mod_down(c, lv, acc, conv, sum, ct_bs, nullptr, ct_bs, 2, 1, bc, true, s, false, &accq, &dq);
        // rescale both components: inverse transform of the last limb, centred remainder to every q_i, forward
        // transform, subtract and divide
        launch_ntt_inv_rows(c, one, XformIO{sum + (uint64_t)(ell - 1) * N, last, (uint64_t)ell * N, N, 2 * bc}, s);
        launch_ntt_inv_cols(c, one, last, N, 2 * bc, c->d_ninv, false, true, s);   // canonical doubles
        launch_rescale_fused(c, lv, sum, last, spread, oc, 2 * bc, s, words32);
    }
    if (merged) return finish(words32 ? "hmult_relin_rescale_merged_u32" : "hmult_relin_rescale_merged");
    return finish(words32 ? "hmult_relin_rescale_u32" : "hmult_relin_rescale");
}

extern "C" int hmult_relin_rescale_merged(const ks_ctx* c, const uint64_t* cta, const uint64_t* ctb, uint32_t ell, const uint64_t* rlk,
                                          uint64_t* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return hmult_impl(c, cta, ctb, ell, rlk, out, batch, ws, ws_bytes, stream, true, false);
}

extern "C" int hmult_relin_rescale(const ks_ctx* c, const uint64_t* cta, const uint64_t* ctb, uint32_t ell, const uint64_t* rlk,
                                   uint64_t* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return hmult_impl(c, cta, ctb, ell, rlk, out, batch, ws, ws_bytes, stream, false, false);
}

extern "C" int hmult_relin_rescale_merged_u32(const ks_ctx* c, const uint32_t* cta, const uint32_t* ctb, uint32_t ell,
                                              const uint32_t* rlk, uint32_t* out, uint32_t batch, void* ws, size_t ws_bytes,
                                              void* stream) {
    return hmult_impl(c, cta, ctb, ell, rlk, out, batch, ws, ws_bytes, stream, true, true);
}

extern "C" int hmult_relin_rescale_u32(const ks_ctx* c, const uint32_t* cta, const uint32_t* ctb, uint32_t ell, const uint32_t* rlk,
                                       uint32_t* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream) {
    return hmult_impl(c, cta, ctb, ell, rlk, out, batch, ws, ws_bytes, stream, false, true);
}
