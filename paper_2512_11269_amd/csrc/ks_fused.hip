// Vertically fused kernels of the key-switching chain (the paper's vertical fusion: dependent limb
// operations on the same positions stay in registers instead of making a round trip through memory).
//
//  * bconv_ntt_cols       base conversion of a digit feeding the column half of the forward transform of
//                         each target limb: the converted limb never exists in memory in coefficient form.
//  * rows_inner_product   row half of the forward transform of every raised limb feeding the inner product
//                         with the key: the raised limb never exists in memory in evaluation form.
//  * rows_moddown_finish  row half of the forward transform of the converted special part feeding
//                         (acc - conv) * P^-1 (+ addend).
//
// Base conversion is coefficient-wise and the column half touches a fixed set of coefficient positions per
// tile, so the first fusion is legal; the inner product and the final scale are slot-wise and the row half
// produces complete slots, so the other two are.
#include "ks_internal.hpp"
#include "ks_tasks.hpp"

namespace ks {

// One source of a conversion: acc[t][k] += y[k] * f[t] as exact integers -- each source point is split once (split3, or
// split2 when every modulus is below 2^32), every target adds PIECES products against its shifted, centred factors.
// REFILL: once y[k] has been consumed, the same registers receive point k of the next source (byte offset next_off in
// the buffer), which then has a whole source's worth of arithmetic to arrive.
// The factors of the next source (fnext: uniform, scalar loads) are requested after the first point, together with
// the limb index of the source after next: scalar loads complete out of order, so the first use of f waits for every
// scalar load in flight, and at that moment only f's own, requested a source ago, should be.
template <int LOG_R, int TS, bool REFILL, int PIECES>
__device__ __forceinline__ void bconv_accumulate(double (&acc)[TS][16], double (&y)[16], const double (&f)[TS][3],
                                                 double (&fnext)[TS][3], const double* const (&hat_row)[TS], int inext,
                                                 uint32_t& limb_after, const uint32_t* src_limb, int iafter, BufferRsrc rsrc,
                                                 uint32_t lane_off, uint32_t next_off) {
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        double y2 = 0.0, y1, y0;
        if constexpr (PIECES == 3) split3(y[k], y2, y1, y0);
        else split2(y[k], y1, y0);
        if (REFILL) y[k] = load_strided_point<LOG_R>(rsrc, lane_off, next_off, k);
#pragma unroll
        for (int tt = 0; tt < TS; ++tt) {
            acc[tt][k] = __builtin_fma(y1, f[tt][1], __builtin_fma(y0, f[tt][0], acc[tt][k]));
            if constexpr (PIECES == 3) acc[tt][k] = __builtin_fma(y2, f[tt][2], acc[tt][k]);
        }
        if (k == 0) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int tt = 0; tt < TS; ++tt)
#pragma unroll
                for (int p = 0; p < PIECES; ++p) fnext[tt][p] = hat_row[tt][inext * 4 + p];
            limb_after = src_limb[iafter];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // one refill per point, in order, each after a point's worth of arithmetic: the wait before point k then leaves 15
    // loads in flight, while the arithmetic of neighbouring points may still interleave
    if (REFILL) {
#pragma unroll
        for (int k = 1; k < 16; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x002, PIECES == 3 ? 6 + 3 * TS : 3 + 2 * TS, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// y: [poly][..][N] canonical doubles y_i = [x_i N^-1 (D/s_i)^-1]_{s_i} (written by ntt_inv_cols with its
// scale table).  Each workgroup owns one column tile (4096 positions) and TS targets of one digit: it
// accumulates sum_i y_i * (D/s_i mod t) as an exact integer (split3) for its 16 positions per thread, then runs the
// column stages of the forward transform modulo t and stores raw doubles.  The sources are re-read by the workgroups of
// the other target subsets; those reads are served by L2 / the last-level cache.
// ------------------------------------------------------------------------------------------------
// PIECES: 3 in general (moduli below 2^36); 2 when every modulus of the context is below 2^32 (the plan's factors are
// then cut at 16 bits: two products per source and target instead of three).
template <int LOG_R, int TS, bool TWO_SETS, int PIECES>
__global__ __launch_bounds__(256) void bconv_ntt_cols(const double* __restrict__ tw, const BConvPlan* __restrict__ plans,
                                                      const uint64_t* __restrict__ y, uint64_t y_ps, uint64_t* __restrict__ out,
                                                      uint64_t out_ps, uint32_t n_subsets) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 1u << (LOG_R - 4), TC = 256 / TILES;
    __shared__ double lds[LOG_R > 4 ? 4096 : 1];
    const uint32_t tid = threadIdx.x, tile = blockIdx.x;
    const uint32_t plan_id = blockIdx.y / n_subsets, subset = blockIdx.y - plan_id * n_subsets;
    const BConvPlan& P = plans[plan_id];
    const int n_dst = (int)P.n_dst, n_src = (int)P.n_src;
    const int t0 = (int)subset * TS;
    if (t0 >= n_dst) return;  // uniform for the whole workgroup
    const uint64_t* yp = y + (uint64_t)blockIdx.z * y_ps;
    uint64_t* op = out + (uint64_t)blockIdx.z * out_ps;
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;

    double acc[TS][16];
#pragma unroll
    for (int tt = 0; tt < TS; ++tt)
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[tt][k] = 0.0;

    // Per-target constants.  They are uniform across the workgroup and travel through scalar loads.
    Mod mt[TS];
    const double* hat_row[TS];
#pragma unroll
    for (int tt = 0; tt < TS; ++tt) {
        const int t = min(t0 + tt, n_dst - 1);  // a ragged last subset recomputes its last target (stored once)
        mt[tt] = P.dst_mod[t];
        hat_row[tt] = &P.hats[t][0][0];
    }

    // Software pipeline over the sources, two per trip so that the uniform factors can alternate between two scalar
    // register sets, with the limb index of the source after next fetched ahead as well: nothing is waited for right
    // after it was requested.  The 16 points of a source are either held in ONE register set that is refilled point by
    // point with the next source while it is consumed (fewer registers; best for the few-workgroup launches of a single
    // ciphertext), or in TWO sets, the idle one filled by a burst of 16 loads (measured 6 % faster on full-chip launches).
    // Sources past the end are zero-padded in the plan (factor 0, a valid limb): prefetches are unconditional -- a
    // conditional one would make the wait-count bookkeeping assume the worst at the join and stall every use on the
    // newest loads -- and an odd source count simply runs one padding source.  Loads are fenced into use order, before
    // the loop as inside it, so that every wait leaves exactly the younger loads in flight.  The points are read through a
    // buffer descriptor of this polynomial's bundle: per-lane offset in a vector register, limb and row offset in a
    // scalar one, so switching limb costs no vector instructions.
    const BufferRsrc ysrd = make_buffer_rsrc(yp, y_ps * 8);
    const uint32_t lane_off = (r0 * 256 + col) * 8;
    double yv[16], ha[TS][3], hb[TS][3];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        yv[k] = load_strided_point<LOG_R>(ysrd, lane_off, P.src_limb[0] * (N * 8), k);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int tt = 0; tt < TS; ++tt)
#pragma unroll
        for (int p = 0; p < PIECES; ++p) ha[tt][p] = hat_row[tt][p];
    uint32_t limb_next = P.src_limb[1];

    if constexpr (!TWO_SETS) {
#pragma unroll 1
        for (int i = 0; i < n_src; i += 2) {
            uint32_t limb_after;
            bconv_accumulate<LOG_R, TS, true, PIECES>(acc, yv, ha, hb, hat_row, min(i + 1, kMaxSrc - 1), limb_after, P.src_limb,
                                              min(i + 2, kMaxSrc - 1), ysrd, lane_off, limb_next * (N * 8));
            bconv_accumulate<LOG_R, TS, true, PIECES>(acc, yv, hb, ha, hat_row, min(i + 2, kMaxSrc - 1), limb_next, P.src_limb,
                                              min(i + 3, kMaxSrc - 1), ysrd, lane_off, limb_after * (N * 8));
        }
    } else {
        double yw[16];
#pragma unroll 1
        for (int i = 0; i < n_src; i += 2) {
            uint32_t limb_after;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                yw[k] = load_strided_point<LOG_R>(ysrd, lane_off, limb_next * (N * 8), k);
                __builtin_amdgcn_sched_barrier(0);
            }
            bconv_accumulate<LOG_R, TS, false, PIECES>(acc, yv, ha, hb, hat_row, min(i + 1, kMaxSrc - 1), limb_after, P.src_limb,
                                               min(i + 2, kMaxSrc - 1), ysrd, lane_off, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                yv[k] = load_strided_point<LOG_R>(ysrd, lane_off, limb_after * (N * 8), k);
                __builtin_amdgcn_sched_barrier(0);
            }
            bconv_accumulate<LOG_R, TS, false, PIECES>(acc, yw, hb, ha, hat_row, min(i + 2, kMaxSrc - 1), limb_next, P.src_limb,
                                               min(i + 3, kMaxSrc - 1), ysrd, lane_off, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // Twiddles are requested one target ahead and always before the previous target's stores are issued: loads and
    // stores share one in-order counter, so a wait for a load issued after a store would also wait for the store to be
    // acknowledged by memory.
    PassTwiddles tws;
    load_col_twiddles<LOG_R>(tws, tw + (size_t)P.dst_mod_id[t0] * N, r0);
#pragma unroll
    for (int tt = 0; tt < TS; ++tt) {
        const int t = t0 + tt;
        if (t < n_dst) {  // uniform
            PassTwiddles cur = tws;
            if (tt + 1 < TS && t + 1 < n_dst) load_col_twiddles<LOG_R>(tws, tw + (size_t)P.dst_mod_id[t + 1] * N, r0);
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[tt][k] = reduce_lazy(acc[tt][k], mt[tt]);
            col_fwd_core<LOG_R>(acc[tt], cur, c, r0, lds, mt[tt]);
            uint64_t* dst = op + (uint64_t)P.dst_limb[t] * N;
#pragma unroll
            for (int k = 0; k < 16; ++k) store_f64(dst + col_row_grouped<LOG_R>(r0, k) * 256 + col, acc[tt][k]);
            if constexpr (LOG_R > 4) __syncthreads();  // the exchange buffer is reused by the next target
        }
    }
}

void launch_bconv_ntt_cols(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const uint64_t* y, uint64_t y_ps,
                           uint64_t* out, uint64_t out_ps, uint32_t n_polys, hipStream_t s, double ops_per_coeff) {
    const uint32_t n_plans = plans.n_plans, max_targets = plans.max_targets;
    const BConvPlan* d_plans = plans.d_plans;
    if (n_polys == 0 || n_plans == 0) return;
    // Which kernel: on launches too small to fill the chip (a single ciphertext) the matrix-core kernel measured 4-5 %
    // faster per key-switch; once a launch has a few workgroups per compute unit the vector kernel wins by 13-24 %.
    const uint32_t tiles16 = 1u << (c->logN - 12);
    const bool small_launch = (uint64_t)tiles16 * n_plans * ((max_targets + 3) / 4) * n_polys < 512;
    const int kernel = c->opt[KS_OPT_BCONV_KERNEL] ? c->opt[KS_OPT_BCONV_KERNEL] : (small_launch && c->logN == 16 ? 2 : 1);
    if (kernel == 2) {
        // algorithmic fp64 / integer vector work per coefficient of this kernel: per target 9 to recombine and reduce the
        // five sums and 35 for the column half; per source 2 to cut it into bytes (the contraction itself runs on the
        // matrix cores: 25 int8 multiply-adds per source and target)
        double vec_ops = 0.0;
        for (uint32_t j = 0; j < n_plans; ++j) vec_ops += plans.meta.plan[j].n_dst * 44.0 + plans.shape_src * 2.0;
        ProfScope ps("bconv_mfma_ntt_cols", (double)limbs_moved_per_poly * n_polys * c->N * 8.0, s, vec_ops * n_polys * c->N);
        const int tl = c->opt[KS_OPT_BCONV_TARGETS] >= 1 && c->opt[KS_OPT_BCONV_TARGETS] <= 3 ? c->opt[KS_OPT_BCONV_TARGETS] : 3;
        launch_bconv_mfma_ntt_cols(c, plans, y, y_ps, out, out_ps, n_polys, tl, s);
        return;
    }
    // Targets per workgroup: fewer targets = more workgroups but more re-reads and re-splits of the sources.  Four (with
    // the two-set source pipeline) is best once the launch has a few workgroups per compute unit; for the
    // single-ciphertext launches three (one-set pipeline) measured best (384 and 256 workgroups: every one resident at
    // once, none waiting for a slot to free up).
    // The context option KS_OPT_BCONV_TARGETS overrides the choice.
    const uint32_t tiles = 1u << (c->logN - 12);
    int ts = (uint64_t)tiles * n_plans * ((max_targets + 3) / 4) * n_polys >= 512 ? 4 : 3;
    if (c->opt[KS_OPT_BCONV_TARGETS] >= 1 && c->opt[KS_OPT_BCONV_TARGETS] <= 4) ts = c->opt[KS_OPT_BCONV_TARGETS];
    if (c->logN != 16 && ts < 3) ts = 3;  // the other ring degrees come with the two production shapes only
    const uint32_t n_subsets = (max_targets + ts - 1) / ts;
    const dim3 grid(tiles, n_plans * n_subsets, n_polys), block(256);
    ProfScope ps("bconv_ntt_cols", (double)limbs_moved_per_poly * n_polys * c->N * 8.0, s, ops_per_coeff * n_polys * c->N);
#define KS_LAUNCH_BCONV(LOGR, TSV)                                                                                                      \
    if (c->pieces == 2)                                                                                                                 \
        hipLaunchKernelGGL((bconv_ntt_cols<LOGR, TSV, (TSV == 4), 2>), grid, block, 0, s, c->d_tw_fwd, d_plans, y, y_ps, out, out_ps,  \
                           n_subsets);                                                                                                  \
    else                                                                                                                                \
        hipLaunchKernelGGL((bconv_ntt_cols<LOGR, TSV, (TSV == 4), 3>), grid, block, 0, s, c->d_tw_fwd, d_plans, y, y_ps, out, out_ps,  \
                           n_subsets)
    if (c->logN == 16) {
        if (ts == 4) { KS_LAUNCH_BCONV(8, 4); }
        else if (ts == 3) { KS_LAUNCH_BCONV(8, 3); }
        else if (ts == 2) { KS_LAUNCH_BCONV(8, 2); }
        else { KS_LAUNCH_BCONV(8, 1); }
    } else {
#define KS_LAUNCH(LOGR)                        \
    if (ts == 4) { KS_LAUNCH_BCONV(LOGR, 4); } \
    else { KS_LAUNCH_BCONV(LOGR, 3); }
        KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
    }
#undef KS_LAUNCH_BCONV
}

// ------------------------------------------------------------------------------------------------
// acc[b][c][pos] = sum_j d~_j[pos] * key[j][c][m(pos)].  For pos inside digit j, d~_j[pos] is the input limb
// itself; otherwise it is the raised limb, whose row half of the forward transform is done here.
// One wavefront = four rows of one limb position; it walks the digits, so d~ is read once and feeds both key
// components (load reuse), and the accumulators are reduced and written once.
// ------------------------------------------------------------------------------------------------
// WD / WK: word types of d and of the key (64-bit, or 32-bit for moduli below 2^32).
template <int LOG_R, typename WD, typename WK, bool PREFETCH>
__global__ __launch_bounds__(64, PREFETCH ? 2 : 0) void rows_inner_product(TwTables tw, TwTables twi,
                                                         const Mod* __restrict__ mods, DigitRanges dg,
                                                         uint32_t ell, uint32_t E, uint32_t L, uint32_t M,
                                                         const WD* __restrict__ d, uint64_t d_ps,
                                                         const uint64_t* __restrict__ lifted, const WK* __restrict__ evk,
                                                         uint64_t* __restrict__ acc, uint32_t* __restrict__ accq_lo,
                                                         uint8_t* __restrict__ accq_hi, uint32_t packed_limbs, uint32_t batch,
                                                         uint32_t special_first) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R;
    __shared__ double lds[4 * kRowPitch];
    __shared__ double lds_ta[4 * 16];
    // Workgroup -> (row group, limb position, batch item).  Consecutive workgroup ids go to the eight XCDs in
    // turn, each with its own L2; the ids that land on one XCD walk through all batch items of one
    // (row group, position) tile before moving to the next tile, so the key slots and twiddles of a tile are
    // fetched into that L2 once and reused by the whole batch.
    const uint32_t slot = blockIdx.x >> 3, b = slot % batch, tile = (slot / batch) * 8 + (blockIdx.x & 7);
    if (tile >= (R / 4) * E) return;  // uniform: padding workgroups when the tile count is not a multiple of 8
    // special_first (launches whose wavefronts are all resident at once, i.e. a single ciphertext): the special limbs take
    // the first workgroup ids.  Their wavefronts have the most arithmetic after their last load (one more transform and the
    // two inverse row passes) and the memory system serves the earliest requests first, so started last they are the tail
    // of the launch (59 k cycles per special wavefront against 37 k for the others; 40.2 -> 37.1 us per launch).  Batched
    // launches keep them last: the next kernel reads exactly these limbs and finds them cached (0.5-2 % per call).
    const uint32_t rg = tile % (R / 4), slot_pos = tile / (R / 4), n_special = E - ell;
    const uint32_t pos = !special_first ? slot_pos : slot_pos < n_special ? ell + slot_pos : slot_pos - n_special;
    task_rows_inner_product<LOG_R, WD, WK, PREFETCH>(tw, twi, mods, dg, ell, E, L, M, d + (uint64_t)b * d_ps, lifted + (uint64_t)b * dg.ndig * E * N, evk,
                                      acc + (uint64_t)b * 2 * E * N, accq_lo + (uint64_t)b * 2 * ell * N,
                                      accq_hi + (uint64_t)b * 2 * ell * N, packed_limbs, pos, rg, threadIdx.x, lds, lds_ta);
}

void launch_rows_inner_product(const ks_ctx* c, const Level& lv, const void* d, uint64_t d_ps, const uint64_t* lifted,
                               const void* evk, uint64_t* acc, uint32_t batch, hipStream_t s, bool d_words32, bool key_words32,
                               const PackedDigits* accq, uint32_t packed_limbs) {
    if (batch == 0) return;
    if (!accq) packed_limbs = 0;
    uint32_t* accq_lo = accq ? accq->lo : nullptr;
    uint8_t* accq_hi = accq ? accq->hi : nullptr;
    DigitRanges dg;
    dg.ndig = lv.ndig;
    for (uint32_t j = 0; j < kMaxDigits; ++j) {
        dg.lo[j] = j < lv.ndig ? lv.digit_lo[j] : 0;
        dg.hi[j] = j < lv.ndig ? lv.digit_hi[j] : 0;
    }
    // reads: every raised digit limb per ciphertext and the key (once per call); writes: both accumulators
    // d (ell limbs per ciphertext) and the key arrive in boundary words, the raised limbs and the sums in 8 bytes
    const double wd = d_words32 ? 0.5 : 1.0, wk = key_words32 ? 0.5 : 1.0;
    ProfScope ps("rows_inner_product",
                 ((double)batch * ((lv.ndig * lv.E - lv.ell) + wd * lv.ell + 2.0 * lv.E - 0.75 * packed_limbs) + wk * 2.0 * lv.ndig * lv.E) *
                     c->N * 8.0,
                 s);
    const uint32_t tiles = (c->N / 1024) * lv.E;
    const dim3 grid(((tiles + 7) / 8) * 8 * batch), block(64);
    // launches with more than two wavefronts per SIMD (1024 SIMDs) to run take the variant that requests the next digit's
    // loads early: 3 % faster there (32.1 -> 31.0 us per multiplication at L = 35); the single-ciphertext launch is bound by
    // bandwidth and gains nothing from it
    const bool prefetch = grid.x > 2048;
#define KS_LAUNCH_IP(LOGR, WDT, WKT, PF)                                                                                           \
    hipLaunchKernelGGL((rows_inner_product<LOGR, WDT, WKT, PF>), grid, block, 0, s, c->tw_fwd, c->tw_inv, c->d_mod, dg, lv.ell, lv.E, c->L, \
                       c->M, static_cast<const WDT*>(d), d_ps, lifted, static_cast<const WKT*>(evk), acc, accq_lo, accq_hi, packed_limbs, batch,   \
                       prefetch ? 0u : 1u)
#define KS_LAUNCH(LOGR)                                                          \
    if (d_words32 && key_words32) KS_LAUNCH_IP(LOGR, uint32_t, uint32_t, false); \
    else if (key_words32) KS_LAUNCH_IP(LOGR, uint64_t, uint32_t, false);         \
    else if (prefetch) KS_LAUNCH_IP(LOGR, uint64_t, uint64_t, true);             \
    else KS_LAUNCH_IP(LOGR, uint64_t, uint64_t, false)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
#undef KS_LAUNCH_IP
}

// ------------------------------------------------------------------------------------------------
// out[b][comp][i] = (acc[b][comp][i] - NTT_rows(conv[b][comp][i])) * P^-1 (+ addend), canonical.
// ------------------------------------------------------------------------------------------------
// ADDEND: 0 = none, 1 = added as it is, 2 = multiplied by addend_mul[i] first.  Compile-time so that the kernel has no
// branch: behind a run-time test every addend load became its own load-wait-use round trip.  A launch covers the
// components comp0 .. comp0 + n_comps - 1 of every batch item.
// ACCP: the ciphertext limbs of the accumulator come packed (acc: [b][2][ell][N] 32-bit low words, acc_hi: the bytes
// above) instead of as the first ell limbs of [b][2][E][N] 64-bit words.
// ADF: format of the addend: 0 = 64-bit words; 1 = packed the same way (addend: [b][2][ell][N] low words, addend_hi: the
// bytes above); 2 = 32-bit words.
template <int LOG_R, bool GATHER, int ADDEND, typename W = uint64_t, bool ACCP = false, int ADF = 0>
__global__ __launch_bounds__(64) void rows_moddown_finish(TwTables tw, const Mod* __restrict__ mods,
                                                          const double* __restrict__ Pinv, const double* __restrict__ addend_mul,
                                                          uint32_t ell, uint32_t E, uint32_t out_limbs,
                                                          const void* __restrict__ acc, const uint8_t* __restrict__ acc_hi,
                                                          const uint64_t* __restrict__ conv,
                                                          W* __restrict__ out, uint64_t out_bs,
                                                          const void* __restrict__ addend, const uint8_t* __restrict__ addend_hi,
                                                          uint64_t addend_bs, uint32_t comp0, uint32_t n_comps, uint32_t galois) {
    constexpr uint32_t N = 256u << LOG_R;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t rg = blockIdx.x, i = blockIdx.y;
    // batch items in descending order: the conversion kernel before this one wrote them in ascending order, so the most
    // recently written ones, still in the last-level cache, are read first (4-5 % on this kernel in batched calls)
    const uint32_t zz = gridDim.z - 1 - blockIdx.z;
    const uint32_t b = zz / n_comps, comp = comp0 + (zz - b * n_comps);
    const void* adp = nullptr;
    const uint8_t* adp_hi = nullptr;
    double admul = 0.0;
    if constexpr (ADDEND != 0) {
        const uint64_t ad_off = (uint64_t)b * addend_bs + ((uint64_t)comp * ell + i) * N;
        if constexpr (ADF == 1) {
            adp = static_cast<const uint32_t*>(addend) + ad_off;
            adp_hi = addend_hi + ad_off;
        } else if constexpr (ADF == 2) {
            adp = static_cast<const uint32_t*>(addend) + ad_off;
        } else {
            adp = static_cast<const uint64_t*>(addend) + ad_off;
        }
    }
    if constexpr (ADDEND == 2) admul = addend_mul[i];
    const uint64_t conv_off = (((uint64_t)b * 2 + comp) * ell + i) * N;
    const void* ap;
    const uint8_t* ap_hi = nullptr;
    if constexpr (ACCP) {
        ap = static_cast<const uint32_t*>(acc) + conv_off;
        ap_hi = acc_hi + conv_off;
    } else {
        ap = static_cast<const uint64_t*>(acc) + (((uint64_t)b * 2 + comp) * E + i) * N;
    }
    task_rows_finish<LOG_R, GATHER, ADDEND, W, ACCP, ADF>(tw, mods[i], i, Pinv[i], admul, conv + conv_off, ap, ap_hi,
                                                          out + (uint64_t)b * out_bs + ((uint64_t)comp * out_limbs + i) * N, adp,
                                                          adp_hi, galois, rg, threadIdx.x, lds);
}

void launch_rows_moddown_finish(const ks_ctx* c, const Level& lv, const uint64_t* acc, const uint64_t* conv, void* out_words,
                                uint64_t out_bs, const void* addend, uint64_t addend_bs, uint32_t addend_comps,
                                uint32_t galois, uint32_t batch, hipStream_t s, const FinishScale* fs, bool out_words32,
                                const PackedDigits* acc_packed, const PackedDigits* addend_packed, bool addend_words32) {
    if (batch == 0) return;
    const void* addend_p = addend_packed ? static_cast<const void*>(addend_packed->lo) : addend;
    const uint8_t* addend_h = addend_packed ? addend_packed->hi : nullptr;
    const double* mul = fs ? fs->mul : c->d_Pinv;
    const double* admul = fs ? fs->addend_mul : nullptr;
    const uint32_t out_limbs = fs ? fs->out_limbs : lv.ell;
    if (out_limbs == 0) return;
    if (!addend_p) addend_comps = 0;
    ProfScope ps("rows_moddown_finish",
                 (double)batch * out_limbs *
                     (2 * 8 + 2 * (acc_packed ? 5 : 8) + (out_words32 ? 1 : 2) * 8 + addend_comps * (addend_packed ? 5 : addend_words32 ? 4 : 8)) * c->N,
                 s);
    const dim3 block(64);
    const uint32_t row_groups = c->N / 1024;
    const void* accp = acc_packed ? static_cast<const void*>(acc_packed->lo) : static_cast<const void*>(acc);
    const uint8_t* acch = acc_packed ? acc_packed->hi : nullptr;
    // one launch for the components that take the addend, one for those that do not
    for (int pass = 0; pass < 2; ++pass) {
        const uint32_t comp0 = pass == 0 ? 0 : addend_comps, n_comps = pass == 0 ? addend_comps : 2 - addend_comps;
        if (n_comps == 0) continue;
        const int mode = pass == 1 ? 0 : (admul ? 2 : 1);
        const dim3 grid(row_groups, out_limbs, batch * n_comps);
#define KS_LAUNCH_FINISH_P(LOGR, GATHER, MODE, WT, ACCP, ADF)                                                                      \
    hipLaunchKernelGGL((rows_moddown_finish<LOGR, GATHER, MODE, WT, ACCP, ADF>), grid, block, 0, s, c->tw_fwd, c->d_mod, mul, admul, \
                       lv.ell, lv.E, out_limbs, accp, acch, conv, static_cast<WT*>(out_words), out_bs, addend_p, addend_h, addend_bs, \
                       comp0, n_comps, galois)
#define KS_LAUNCH_FINISH(LOGR, GATHER, MODE, WT, ACCP) KS_LAUNCH_FINISH_P(LOGR, GATHER, MODE, WT, ACCP, 0)
    // a packed addend comes with a packed accumulator (multiplications); an addend in 32-bit words with a packed accumulator
    // and 32-bit output (hoisted rotations in 32-bit words)
#define KS_LAUNCH_MODES(LOGR, WT)                                                        \
    if (addend_packed && mode != 0) {                                                    \
        if (mode == 2) KS_LAUNCH_FINISH_P(LOGR, false, 2, WT, true, 1);                  \
        else KS_LAUNCH_FINISH_P(LOGR, false, 1, WT, true, 1);                            \
    } else if (addend_words32 && mode != 0) {                                            \
        if (galois == 1) KS_LAUNCH_FINISH_P(LOGR, false, 1, uint32_t, true, 2);          \
        else KS_LAUNCH_FINISH_P(LOGR, true, 1, uint32_t, true, 2);                       \
    } else if (acc_packed) {                                                             \
        if (mode == 0) KS_LAUNCH_FINISH(LOGR, false, 0, WT, true);                       \
        else if (mode == 2) KS_LAUNCH_FINISH(LOGR, false, 2, WT, true);                  \
        else if (galois == 1) KS_LAUNCH_FINISH(LOGR, false, 1, WT, true);                \
        else KS_LAUNCH_FINISH(LOGR, true, 1, WT, true);                                  \
    } else if (mode == 0) KS_LAUNCH_FINISH(LOGR, false, 0, WT, false);                   \
    else if (mode == 2) KS_LAUNCH_FINISH(LOGR, false, 2, WT, false);                     \
    else if (galois == 1) KS_LAUNCH_FINISH(LOGR, false, 1, WT, false);                   \
    else KS_LAUNCH_FINISH(LOGR, true, 1, WT, false)
#define KS_LAUNCH(LOGR)                                     \
    if (out_words32) { KS_LAUNCH_MODES(LOGR, uint32_t); }   \
    else { KS_LAUNCH_MODES(LOGR, uint64_t); }
        KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
#undef KS_LAUNCH_MODES
#undef KS_LAUNCH_FINISH
#undef KS_LAUNCH_FINISH_P
    }
}

// ------------------------------------------------------------------------------------------------
// Rescale, first half: the centred remainder of the dropped limb (coefficient domain, canonical doubles) is
// reduced modulo q_i and sent straight through the column half of NTT_{q_i}; the "spread" limbs never exist
// in coefficient form.  last: [polys][N]; out: [polys][ell-1][N] raw doubles.
// ------------------------------------------------------------------------------------------------
template <int LOG_R>
__global__ __launch_bounds__(256) void rescale_cols(const double* __restrict__ tw, const Mod* __restrict__ mods, uint32_t ell,
                                                    const uint64_t* __restrict__ last, uint64_t* __restrict__ out) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 1u << (LOG_R - 4), TC = 256 / TILES;
    __shared__ double lds[LOG_R > 4 ? 4096 : 1];
    const uint32_t tid = threadIdx.x, tile = blockIdx.x, i = blockIdx.y, p = blockIdx.z;
    const Mod m = mods[i];
    const double ql = mods[ell - 1].p, half = (ql - 1.0) * 0.5;
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;
    const uint64_t* src = last + (uint64_t)p * N;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load_f64(src + col_row_strided<LOG_R>(r0, k) * 256 + col);
    load_col_twiddles<LOG_R>(t, tw + (size_t)i * N, r0);
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = reduce_lazy(v[k] > half ? v[k] - ql : v[k], m);
    col_fwd_core<LOG_R>(v, t, c, r0, lds, m);
    uint64_t* dst = out + ((uint64_t)p * (ell - 1) + i) * N;
#pragma unroll
    for (int k = 0; k < 16; ++k) store_f64(dst + col_row_grouped<LOG_R>(r0, k) * 256 + col, v[k]);
}

// Rescale, second half: row half of the forward transform, then out = (x - w) * q_{ell-1}^-1 mod q_i.
// x: [polys][ell][N] canonical; spread: [polys][ell-1][N] raw doubles; out: [polys][ell-1][N] canonical.
template <int LOG_R, typename W>
__global__ __launch_bounds__(64) void rows_rescale_finish(TwTables tw, const Mod* __restrict__ mods,
                                                          const double* __restrict__ qlinv, uint32_t ell,
                                                          const uint64_t* __restrict__ x, const uint64_t* __restrict__ spread,
                                                          W* __restrict__ out) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t tid = threadIdx.x, rg = blockIdx.x, i = blockIdx.y, p = blockIdx.z;
    const Mod m = mods[i];
    const double scale = qlinv[i];
    const uint32_t j0 = tid & 15, rr = tid >> 4, row = rg * 4 + rr;
    const uint32_t off = row * 256 + j0;
    const uint64_t* src = spread + ((uint64_t)p * (ell - 1) + i) * N + off;
    const uint64_t* xp = x + ((uint64_t)p * ell + i) * N + off;
    W* op = out + ((uint64_t)p * (ell - 1) + i) * N + off;
    double w[16], a[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) w[k] = load_f64(src + 16 * k);
#pragma unroll
    for (int k = 0; k < 16; ++k) a[k] = u64_to_f64(xp[16 * k]);
    load_row_twiddles(t, tw, i, N, R + row, j0, m);
    row_fwd_core(w, t, j0, lds + rr * kRowPitch, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) op[16 * k] = f64_to_word<W>(canon(mulmod_lazy(a[k] - w[k], scale, m), m));
}

void launch_rescale_fused(const ks_ctx* c, const Level& lv, const uint64_t* x, const uint64_t* last, uint64_t* spread,
                          void* out, uint32_t n_polys, hipStream_t s, bool out_words32) {
    if (n_polys == 0 || lv.ell < 2) return;
    const uint32_t nl = lv.ell - 1;
    {
        ProfScope ps("rescale_cols", ((double)n_polys * (1 + nl)) * c->N * 8.0, s);
#define KS_LAUNCH(LOGR) \
    hipLaunchKernelGGL(rescale_cols<LOGR>, dim3(1u << (LOGR - 4), nl, n_polys), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, lv.ell, last, spread)
        KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
    }
    {
        ProfScope ps("rows_rescale_finish", (double)n_polys * nl * (out_words32 ? 2.5 : 3.0) * c->N * 8.0, s);
#define KS_LAUNCH(LOGR)                                                                                                                      \
    if (out_words32)                                                                                                                         \
        hipLaunchKernelGGL((rows_rescale_finish<LOGR, uint32_t>), dim3(1u << (LOGR - 2), nl, n_polys), dim3(64), 0, s, c->tw_fwd, c->d_mod,   \
                           lv.d_qlinv, lv.ell, x, spread, static_cast<uint32_t*>(out));                                                      \
    else                                                                                                                                     \
        hipLaunchKernelGGL((rows_rescale_finish<LOGR, uint64_t>), dim3(1u << (LOGR - 2), nl, n_polys), dim3(64), 0, s, c->tw_fwd, c->d_mod,   \
                           lv.d_qlinv, lv.ell, x, spread, static_cast<uint64_t*>(out))
        KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
    }
}

}  // namespace ks
