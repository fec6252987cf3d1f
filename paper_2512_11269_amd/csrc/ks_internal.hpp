// Internal declarations shared by the translation units of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <mutex>
#include <vector>

#include "../../include/ks.h"
#include "ks_device.hpp"
#include "ks_tiles.hpp"

namespace ks {

constexpr int kMaxSrc = 16;     // source limbs of one base conversion (alpha or K)
constexpr int kMfmaSlots = 6;   // 16-byte operand slots of the matrix-core conversion: 3 instructions x 2 lane halves, 3 sources each
constexpr int kMfmaPlanes = 5;  // signed base-256 digits of a 36-bit residue or factor
constexpr int kMaxDst = 256;    // target limbs of one base conversion
constexpr int kMaxLimbs = 192;  // limbs of one polynomial bundle addressed by a LimbMap
constexpr int kMaxDigits = 8;

// Which limbs of a polynomial bundle a transform launch touches: limb `idx` lives at element offset
// off[idx] * N from the bundle's base and is taken modulo moduli[mod[idx]].  Passed by value.
struct LimbMap {
    uint16_t off[kMaxLimbs];
    uint8_t mod[kMaxLimbs];
    uint32_t n;
};

// Constants of one fast base conversion, read by the kernel through uniform (scalar) loads.
struct BConvPlan {
    uint32_t n_src, n_dst;
    uint32_t src_limb[kMaxSrc];  // limb index inside the input bundle (32-bit fields: scalar loads)
    uint32_t dst_limb[kMaxDst];  // limb index inside the output bundle
    Mod src_mod[kMaxSrc];
    double src_inv[kMaxSrc];     // (D / s_i)^-1 mod s_i
    Mod dst_mod[kMaxDst];
    uint32_t dst_mod_id[kMaxDst];  // modulus id of each target (selects its twiddle table)
    // hat3[t][i][k], k = 0..2: the three 12-bit pieces (low to high) of (D / s_i) mod t.  A 36-bit residue times a
    // 12-bit piece is below 2^48, so up to 16 such products add up exactly in a double: the conversion sum costs
    // three FMAs per source and target plus one short recombination per target instead of a full modular product.
    double hat3[kMaxDst][kMaxSrc][3];
    // hats[t][i][k], k = 0..2: centred([(D / s_i) 2^(12 k)]_t) * 2^(-12 k), the factors that go with the three pieces
    // of a split source residue (split3); [3] pads the row to 32 bytes.  Zero for padding sources.
    double hats[kMaxDst][kMaxSrc][4];
    // Matrix-core form (int8 MFMA, see ks_bconv_mfma.hip).  A source residue y = sum_a d_a 256^a is cut into five signed
    // digits; for every digit position a the factor F_a = centred([(D / s_i) 256^a]_t) is cut the same way into digits
    // e_b, so that y (D / s_i) = sum_b 256^b sum_a d_a e_{a,b} (mod t): five small integer sums per target, each a dot
    // product over (source, a) that the matrix cores accumulate exactly in 32 bits.
    // The sources are dealt to operand slots of 16 bytes, mfma_nps (1..3) sources per slot, slot = 2 * instruction + lane
    // half; inside a slot, bytes 4 e + a (a < 4) belong to digit a of the slot's e-th source and byte 12 + e to its digit 4.
    // afac[t][b][slot] is the A-operand row of target t, digit plane b, in that byte order (zero where a slot has no source).
    uint32_t mfma_nm, mfma_nps;                 // instructions per block (1..3), sources per slot
    uint32_t mfma_src_limb[kMfmaSlots * 3];     // limb of slot-major source k (padding: the first source's limb)
    alignas(16) int8_t afac[kMaxDst][kMfmaPlanes][kMfmaSlots][16];
    // everything the matrix-core kernel needs to know about a target, in one 32-byte record (one load per lane)
    struct alignas(32) TargetRec {
        Mod m;
        uint32_t mod_id, limb, pad[2];
    } trec[kMaxDst];
};

// The part of a plan a kernel launch carries by value in its arguments (no dependent load before the first source
// read): target count and source limbs in operand-slot order.
struct PlanMeta {
    uint32_t n_dst;
    uint32_t src_limb[kMfmaSlots * 3];
};
struct LaunchMeta {
    PlanMeta plan[kMaxDigits];
};
// The plans of one conversion launch (one per digit for ModUp, a single one otherwise): device copies plus the host
// facts the launchers need.
struct PlanSet {
    BConvPlan* d_plans = nullptr;  // [n_plans] device
    uint32_t n_plans = 0;
    uint32_t max_targets = 0;      // largest target count of a plan
    uint32_t shape_src = 0;        // source count the matrix-core operand slots were laid out for (the largest of the plans)
    LaunchMeta meta{};
};

// Everything the key-switching pipeline needs at one level ell.
struct Level {
    uint32_t ell = 0, ndig = 0, E = 0;     // E = ell + K extended limb count
    uint32_t n_new = 0;                    // sum over digits of (E - alpha_j): limbs produced by ModUp
    PlanSet modup;                         // one plan per digit
    PlanSet moddown;
    LimbMap lifted_map;                    // new limbs inside the [ndig][E][N] lifted bundle
    LimbMap special_map;                   // the K special limbs inside an [E][N] accumulator
    LimbMap q_map;                         // limbs 0..ell-1, modulus id = limb index
    uint32_t digit_lo[kMaxDigits], digit_hi[kMaxDigits];
    double* d_qlinv = nullptr;             // [ell-1] device: q_{ell-1}^-1 mod q_i (rescale)
    double* d_modup_scale = nullptr;       // [ell] device: N^-1 (D_j / q_i)^-1 mod q_i, j = digit of limb i
    // ModDown merged with rescale: one conversion from {p_0..p_{K-1}, q_{ell-1}} (product D) to q_0..q_{ell-2}
    PlanSet merged;                        // d_plans == nullptr when unavailable (ell < 2 or K + 1 sources too many)
    LimbMap merged_map;                    // the K special limbs and limb ell-1 inside an [E][N] accumulator
    LimbMap last_map;                      // limb ell-1 alone
    double* d_merged_scale = nullptr;      // [K+1] device: N^-1 (D / s)^-1 mod s, s in merged_map order
    double* d_Dinv = nullptr;              // [ell-1] device: D^-1 mod q_i
    double Pmod_last = 0.0;                // P mod q_{ell-1}
};

}  // namespace ks

struct ks_ctx {
    int device = 0;
    uint32_t logN = 0, N = 0, L = 0, K = 0, dnum = 0, alpha = 0, M = 0;
    std::vector<uint64_t> mod, psi;       // host copies, index = modulus id
    ks::Mod* d_mod = nullptr;             // [M]
    double* d_ninv = nullptr;             // [M]  N^-1 mod m
    double* d_Pinv = nullptr;             // [L]  P^-1 mod q_i
    double* d_Pmod = nullptr;             // [L]  P mod q_i
    uint64_t* d_one = nullptr;            // [2]  the residue 1 (unit plaintext slot)
    double* d_moddown_scale = nullptr;    // [K]  N^-1 (P / p_k)^-1 mod p_k
    double* d_tw_fwd = nullptr;           // [M][N] psi^brv(k)
    double* d_tw_inv = nullptr;           // [M][N] psi^-brv(k)
    double* d_trow = nullptr;             // [2][M][N/16] compact last-pass generators, forward then inverse
    double* d_w16 = nullptr;              // [2][M][8] powers of the primitive 16th root, forward then inverse
    ks::TwTables tw_fwd{}, tw_inv{};      // the three tables of each direction bundled for the row kernels
    std::vector<ks::Level> levels;        // index ell-1
    int opt[KS_OPT_COUNT_] = {};          // ks_ctx_set_option values, index = option id
    int pieces = 3;                       // pieces a source residue is cut into by the fused conversion: 2 iff every modulus < 2^32
    mutable std::mutex mu;
    mutable std::map<std::vector<uint32_t>, ks::PlanSet> bconv_cache;  // key: n_src, src ids, dst ids
};

namespace ks {

// ---- host number theory (ks_ctx.hip) ----
uint64_t h_mulmod(uint64_t a, uint64_t b, uint64_t m);
uint64_t h_powmod(uint64_t a, uint64_t e, uint64_t m);
uint64_t h_invmod(uint64_t a, uint64_t m);
// shape_src: the source count that fixes the operand-slot layout of the matrix-core tables (all plans of one launch must
// agree on it); 0 = n_src.
void fill_bconv_plan(const ks_ctx* c, BConvPlan* plan, const uint32_t* src_ids, const uint16_t* src_limb, uint32_t n_src,
                     const uint32_t* dst_ids, const uint16_t* dst_limb, uint32_t n_dst, uint32_t shape_src = 0);

// thread-local HIP error text
void set_hip_error(hipError_t e, const char* where);

// Optional per-kernel timing (ks_profile_enable): when on, every launcher brackets its kernel with a pair of
// HIP events on the launch stream and books the kernel's algorithmic bytes (what it must read plus write).
struct ProfScope {
    // ops: algorithmic fp64 vector instructions per lane (FMA, MUL, ADD and RNDNE each count one)
    ProfScope(const char* name, double bytes, hipStream_t s, double ops = 0.0);
    ~ProfScope();
    int slot;
    hipStream_t stream;
};

// Dispatch on the ring degree: N = 2^12 .. 2^16 <-> R = N / 256 = 2^4 .. 2^8 rows.
#define KS_FOR_LOG_R(logN, M) \
    switch (logN) {           \
        case 12: M(4); break; \
        case 13: M(5); break; \
        case 14: M(6); break; \
        case 15: M(7); break; \
        default: M(8); break; \
    }

// ---- launchers: all asynchronous on `s`, no allocation ----
// In/out element formats of the two-phase transform.  Intermediate results between the two phases are
// stored as raw doubles (lazy representatives) in the same 8-byte slots.
struct XformIO {
    const void* in;
    void* out;
    uint64_t in_poly_stride, out_poly_stride;  // elements between consecutive bundles
    uint32_t n_polys;
};
// forward: coefficient (canonical u64) -> evaluation (canonical u64)
void launch_ntt_fwd(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s);
// inverse: evaluation (canonical u64) -> coefficient (canonical u64)
void launch_ntt_inv(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s);
// both directions on limbs in 32-bit words, in place (canonical residues between the two passes as well)
void launch_ntt_u32(const ks_ctx* c, const LimbMap& map, uint32_t* data, uint64_t ps_words, uint32_t n_polys, bool inverse,
                    hipStream_t s);
// The two halves of each transform on their own (the fused pipeline replaces some halves by fused kernels).
void launch_ntt_fwd_cols(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s);
void launch_ntt_fwd_rows(const ks_ctx* c, const LimbMap& map, uint64_t* data, uint64_t ps_words, uint32_t n_polys, hipStream_t s);
// in_words32: io.in holds 32-bit words (strides still count elements)
void launch_ntt_inv_rows(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s, bool in_words32 = false);
// scale_tab: multiplier applied with the final reduction, indexed by the limb's position in `map` (scale_by_idx)
// or by its modulus id; out_f64: leave the canonical result as a double for a following fused kernel.
void launch_ntt_inv_cols(const ks_ctx* c, const LimbMap& map, uint64_t* data, uint64_t ps_words, uint32_t n_polys,
                         const double* scale_tab, bool scale_by_idx, bool out_f64, hipStream_t s);

// Fused base conversion + column half of the forward transform.  y: pre-scaled canonical doubles
// y_i = [x_i N^-1 (D/s_i)^-1]; out: raw doubles ready for the row half.  One plan per blockIdx.y group.
void launch_bconv_ntt_cols(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const uint64_t* y, uint64_t y_ps,
                           uint64_t* out, uint64_t out_ps, uint32_t n_polys, hipStream_t s, double ops_per_coeff = 0.0);
// The same conversion + column half on the matrix cores (ks_bconv_mfma.hip); tl = targets per lane half, 1..3.
void launch_bconv_mfma_ntt_cols(const ks_ctx* c, const PlanSet& plans, const uint64_t* y, uint64_t y_ps, uint64_t* out,
                                uint64_t out_ps, uint32_t n_polys, int tl, hipStream_t s);
// Upload host plans as a PlanSet (allocates; ks_ctx_create and bconv plan registration only).  Returns a HIP error code.
hipError_t upload_plans(const BConvPlan* host_plans, uint32_t n_plans, uint32_t shape_src, PlanSet* out);
// Canonical residues in packed form: bits 0..31 in lo, the bits above (moduli are below 2^36) in hi, both with the
// element index of the tensor they stand for; 5 bytes a residue instead of 8.  The hoisted rotations keep the finished
// raised digits ([b][ndig][E][N], what their gathers read) and the ciphertext limbs of their accumulators this way.
struct PackedDigits {
    uint32_t* lo;
    uint8_t* hi;
};
// Fused row half of the forward transform of the raised digits + inner product with the key.
// d_words32 / key_words32: d / the key hold one residue per 32-bit word (d_words32 implies key_words32)
// accq != nullptr: the first packed_limbs ciphertext limbs of the sums go to accq ([b][2][ell][N], packed) instead of acc.
void launch_rows_inner_product(const ks_ctx* c, const Level& lv, const void* d, uint64_t d_ps, const uint64_t* lifted,
                               const void* evk, uint64_t* acc, uint32_t batch, hipStream_t s, bool d_words32 = false,
                               bool key_words32 = false, const PackedDigits* accq = nullptr, uint32_t packed_limbs = 0);
// Fused row half of the forward transform of the converted limbs + (acc - conv) P^-1 (+ addend).
// fs == nullptr: multiply by P^-1, addend unscaled, ell output limbs.  Otherwise (merged ModDown + rescale): multiply by
// fs->mul[i], scale the addend by fs->addend_mul[i], and write only the first fs->out_limbs limbs per component.
// acc_packed: the ciphertext limbs of the accumulator are read from there ([b][2][ell][N]) instead of from acc.
// addend_packed (with acc_packed, galois == 1): the addend is read from there ([b][2][ell][N], addend_batch_stride in
// elements) instead of from addend.  addend_words32 (with acc_packed and out_words32): addend holds 32-bit words.
struct FinishScale {
    const double* mul;
    const double* addend_mul;
    uint32_t out_limbs;
};
void launch_rows_moddown_finish(const ks_ctx* c, const Level& lv, const uint64_t* acc, const uint64_t* conv, void* out,
                                uint64_t out_batch_stride, const void* addend, uint64_t addend_batch_stride,
                                uint32_t addend_comps, uint32_t galois, uint32_t batch, hipStream_t s,
                                const FinishScale* fs = nullptr, bool out_words32 = false, const PackedDigits* acc_packed = nullptr,
                                const PackedDigits* addend_packed = nullptr, bool addend_words32 = false);
// acc[b][comp][limb] += mul * addend[b][comp][limb] for one ciphertext limb of both components (canonical in, canonical
// out); addend: [b][2][ell][N] packed
void launch_add_scaled_limb(const ks_ctx* c, uint64_t* acc, uint64_t acc_ps, const PackedDigits& addend, uint32_t ell, uint32_t limb,
                            double mul, uint32_t batch, hipStream_t s);

// Fused rescale: last = coefficient-domain dropped limb as canonical doubles [polys][N]; spread = scratch
// [polys][ell-1][N]; out[p][i] = (x[p][i] - NTT(centred last mod q_i)) * q_{ell-1}^-1.
void launch_rescale_fused(const ks_ctx* c, const Level& lv, const uint64_t* x, const uint64_t* last, uint64_t* spread,
                          void* out, uint32_t n_polys, hipStream_t s, bool out_words32 = false);

// words32: in and out hold one residue per 32-bit word (strides in words either way)
void launch_bconv(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const void* in, uint64_t in_poly_stride,
                  void* out, uint64_t out_poly_stride, uint32_t n_polys, hipStream_t s, bool words32 = false);
// the same conversion on the matrix cores (ks_bconv_mfma.hip)
void launch_bconv_mfma(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const uint64_t* in, uint64_t in_poly_stride,
                       uint64_t* out, uint64_t out_poly_stride, uint32_t n_polys, hipStream_t s);

// Rotations handled by one launch of the gather kernels (more are chained).
constexpr int kMacRotations = 16;
struct MacRotations {
    uint32_t n;
    uint32_t galois[kMacRotations];
    const void* key[kMacRotations];  // [dnum][2][L+K][N], 64- or 32-bit words
    const void* pt[kMacRotations];   // [L+K][N], same word size as the keys
};
// What the sigma_g gathers of a rotation read: the bundle [b][ndig][E][N] of the finished raised digits with, in the slots
// of a digit's own positions, the limbs of the polynomial itself.  hi != nullptr: packed residues (lo, hi); hi == nullptr:
// 32-bit words in lo (moduli below 2^32).
struct GatherSources {
    const uint32_t* lo;
    const uint8_t* hi;
};
// Finish the bundle in one launch: the row half of the forward transform of the raised limbs (`lifted`, the bundle's
// element layout, raw doubles after the column half) and a copy of the polynomials' own limbs d[b][pos] (64-bit words with
// a packed bundle, 32-bit words with a 32-bit one; d_ps words apart) into the slots (b, digit of pos, pos).
// out.hi == nullptr: a bundle of 32-bit words.
void launch_gather_bundle_rows(const ks_ctx* c, const Level& lv, const uint64_t* lifted, const void* d, uint64_t d_ps, bool d_words32,
                               const PackedDigits& out, uint32_t n_polys, hipStream_t s);

// acc[r][b][c][pos] = sum_j sigma_{g_r}(src_j)[pos] * key_r[j][c][ext_id(pos)] for every rotation r of `rot` (pt unused);
// src_j[pos] = d[b][pos] when pos lies in digit j, otherwise lifted[b][j][pos]: slot (b, j, pos) of the bundle `src`.
// key_words32: keys (and plaintexts) hold one residue per 32-bit word; 32-bit sources imply 32-bit keys.
// The special limbs of the result go to acc ([r][b][2][E][N], ciphertext limbs left untouched), the ciphertext limbs to
// accq ([r][b][2][ell][N], packed).
void launch_inner_product(const ks_ctx* c, const Level& lv, const GatherSources& src, const MacRotations& rot, uint64_t* acc,
                          const PackedDigits& accq, uint32_t batch, hipStream_t s, bool key_words32 = false);

// u[b][c][pos] (+)= sum_r pt_r[pos] * (sum_j sigma_r(src_j)[pos] key_r[j][c][pos] + [c = 0][pos < ell] P sigma_r(c0)[pos]);
// ct: [b][2][ell][N] (c0, c1) in 64-bit words with packed sources, in 32-bit words with 32-bit sources (ct_bs in words);
// src: c1 and its finished raised digits.  accumulate: add to what u already holds.
// galois[r] == 1: the term is P (c0, c1) and key[r] is not read; pt[r] == nullptr: the constant 1.
void launch_rotate_mac(const ks_ctx* c, const Level& lv, const void* ct, uint64_t ct_bs, const GatherSources& src,
                       const MacRotations& rot, uint64_t* u, uint32_t batch, bool accumulate, hipStream_t s, bool key_words32 = false);

// The key-switch chain behind ks_keyswitch / ks_keyswitch_u32 (argument checks included); ws is any device buffer of
// at least ks_workspace_bytes(KS_OP_KEYSWITCH) bytes, whose contents need no initialisation.
int keyswitch_impl(const ks_ctx* c, const void* d, uint32_t ell, const void* evk, void* out, uint32_t batch, void* ws,
                   size_t ws_bytes, void* stream, bool words32);

// Resolve this device's copy of the library-owned static scratch array (ks_static.hip); called by ks_ctx_create with
// the device current.  Returns a HIP error code.
hipError_t bind_static_scratch(int device);

// d0 = b1 b2, d1 = a1 b2 + a2 b1 -> dq [batch][2][ell][N] packed; d2 = a1 a2 -> d2 [batch][ell][N] 64-bit words
void launch_tensor_product(const ks_ctx* c, const void* cta, const void* ctb, uint64_t* d2, const PackedDigits& dq, uint32_t ell,
                           uint32_t batch, hipStream_t s, bool in_words32 = false);
}  // namespace ks
