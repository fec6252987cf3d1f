// The bodies of the pipeline kernels as device functions over explicit tile coordinates (the kernels in ks_ntt.hip,
// ks_fused.hip and ks_bconv_mfma.hip map their block indices onto them).  "Wave tasks" are executed by one wavefront (lane = threadIdx.x % 64) on four 256-point rows and need
// 4 * kRowPitch doubles of LDS of their own; "workgroup tasks" are executed by 256 threads on a column tile.
// Every task contains the same number of workgroup barriers for all its threads.
#pragma once
#include "ks_internal.hpp"
#include "ks_tiles.hpp"

namespace ks {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---- inverse transform, row half: canonical residues in (64- or 32-bit words), raw doubles out (|x| <= 0.501 p) ----
// ip / op: the limb's first element; rg: group of four rows; lds_wave: 4 * kRowPitch doubles.
template <int LOG_R, typename W>
__device__ __forceinline__ void task_inv_rows(const TwTables& twi, Mod m, uint32_t mod_id, const W* ip,
                                              uint64_t* op, uint32_t rg, uint32_t lane, double* lds_wave) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R;
    const uint32_t j0 = lane & 15, rr = lane >> 4, row = rg * 4 + rr;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = word_to_f64<W>(ip[row * 256 + j0 + 16 * k]);
    load_row_twiddles(t, twi, mod_id, N, R + row, j0, m);
    row_inv_core(v, t, j0, lds_wave + rr * kRowPitch, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) store_f64(op + row * 256 + j0 + 16 * k, v[k]);
}

// ---- inverse transform, column half, in place or not: raw doubles in; out = canonical [x * scale]_m --------------------
// Wi: the modulus's inverse twiddle table; tile: TC columns; tid < TC * R / 16; lds: TC * R doubles.
template <int LOG_R, int TC, bool OUT_F64>
__device__ __forceinline__ void task_inv_cols(const double* __restrict__ Wi, Mod m, double scale, const uint64_t* in, uint64_t* out,
                                              uint32_t tile, uint32_t tid, double* lds) {
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load_f64(in + col_row_grouped<LOG_R>(r0, k) * 256 + col);
    load_col_twiddles<LOG_R>(t, Wi, r0);
    col_inv_core<LOG_R, TC>(v, t, c, r0, lds, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const double r = canon(mulmod_lazy(v[k], scale, m), m);
        uint64_t* dst = out + col_row_strided<LOG_R>(r0, k) * 256 + col;
        if constexpr (OUT_F64) store_f64(dst, r);
        else *dst = f64_to_u64(r);
    }
}

// ---- base conversion on the matrix cores + column half of the forward transform (see ks_bconv_mfma.hip) --------------
// Adding 2^52 + 0x80808080 to a canonical residue y < 2^36 (held as a double) leaves y + 0x80808080 in the mantissa:
// its low four bytes, each with the top bit flipped, are the signed digits d_0..d_3 (digit = byte - 128), and bits
// 32..39 are the non-negative digit d_4 <= 16.
constexpr double kDigitBias = 4503599627370496.0 + 2155905152.0;

// Twiddles of the column butterflies, staged in LDS (both lane halves of a workgroup need different tables, so they
// cannot ride in scalar registers, and 30 vector registers per target would cost a wavefront of occupancy):
//   first pass : entries 1..15 = W[j], the sub-tree below heap node 1, the same for every thread of a half;
//   second pass: for every row group r0, entries (1 << ul) + g = W[(1 << (E + ul)) + (r0 << ul) + g] for the last E local
//                stages ul = 4 - E .. 3 (for E = 4 the sub-tree below node 16 + r0).
// Layout per (half, target): [1 + S][16] doubles, S = R / 16 row groups.
template <int LOG_R>
__device__ __forceinline__ uint32_t col_twiddle_index(uint32_t slot, uint32_t j) {
    constexpr int E = LOG_R - 4;
    if (j == 0) return 0;
    if (slot == 0) return j;
    const uint32_t ul = 31u - __clz(j), g = j - (1u << ul), r0 = slot - 1;
    return (int)ul >= 4 - E ? (1u << (E + ul)) + (r0 << ul) + g : 0u;
}

template <int LOG_R, int TL>
struct MfmaConvShape {
    static constexpr uint32_t R = 1u << LOG_R, TC = 2048u >> LOG_R;  // tile: TC columns x R rows = 2048 positions
    static constexpr int E = LOG_R - 4, S = 1 << E;
    // exchange buffer of the column butterflies, one region per lane half; rows are padded so that the 16-row groups the
    // second pass reads start in different banks
    static constexpr uint32_t PADW = TC <= 16 ? TC : 0, HALF_WORDS = R * TC + (R / 16) * PADW;
    static constexpr uint32_t TW_WORDS = (1 + S) * 16;  // per (half, target)
    static constexpr uint32_t LDS_WORDS = LOG_R > 4 ? 2 * HALF_WORDS : 1, LDS_TW_WORDS = 2 * TL * TW_WORDS;
};

// 256 threads; yp / y_bytes: the source bundle of this polynomial; op: its output bundle; tile: 2048 positions;
// t0: first of the 2 TL targets (t0 < n_dst); lds: LDS_WORDS doubles; lds_tw: LDS_TW_WORDS doubles.
template <int LOG_R, int TL, int NM, int NPS>
__device__ __forceinline__ void task_bconv_mfma_cols(const double* __restrict__ tw, const BConvPlan& P, const PlanMeta& PM,
                                                     const uint64_t* __restrict__ yp, uint64_t y_bytes, uint64_t* __restrict__ op,
                                                     uint32_t tile, int t0, uint32_t tid, double* lds, double* lds_tw) {
    using Shape = MfmaConvShape<LOG_R, TL>;
    constexpr uint32_t N = 256u << LOG_R, TC = Shape::TC, PADW = Shape::PADW, HALF_WORDS = Shape::HALF_WORDS, TW_WORDS = Shape::TW_WORDS;
    constexpr int E = Shape::E, S = Shape::S;
    const uint32_t lane = tid & 63u, h = lane >> 5, p = (tid >> 6) * 32u + (lane & 31u);
    const uint32_t c = p & (TC - 1), r0 = p / TC, col = tile * TC + c;
    const int n_dst = (int)PM.n_dst;

    // B operand: the sources of this lane's slots, read through a buffer descriptor (per-lane offset = position + limb).
    // The first positions are requested before anything else.
    const BufferRsrc ysrd = make_buffer_rsrc(yp, y_bytes);
    uint32_t voff[NM][NPS];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int e = 0; e < NPS; ++e) {
            // both candidates through scalar registers (a select between two loads would become one per-lane load)
            const uint32_t limb0 = __builtin_amdgcn_readfirstlane(PM.src_limb[(2 * m) * NPS + e]);
            const uint32_t limb1 = __builtin_amdgcn_readfirstlane(PM.src_limb[(2 * m + 1) * NPS + e]);
            const uint32_t limb = h ? limb1 : limb0;
            voff[m][e] = (limb * N + r0 * 256 + col) * 8;
        }
    constexpr uint32_t kStrideBytes = (16u << LOG_R) * 8u;  // rows r0 + (R / 16) k
    // positions whose loads are in flight together, and whether position k - 1 is recombined under the matrix instructions
    // of position k (a second set of result registers) or right away: the single-target shape is kept within 128 registers
    constexpr int kLoadBudget = TL == 1 ? 16 : 32;  // source values a lane keeps in flight
    constexpr int KB = kLoadBudget / (NM * NPS) >= 16 ? 16 : kLoadBudget / (NM * NPS) >= 1 ? kLoadBudget / (NM * NPS) : 1;
    constexpr bool OVERLAP = TL > 1;
    double yv[KB][NM][NPS];
#pragma unroll
    for (int kk = 0; kk < KB; ++kk)
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int e = 0; e < NPS; ++e)
                yv[kk][m][e] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(ysrd, (int)voff[m][e], (int)(kk * kStrideBytes), 0));

    // A operand: this lane's row of the factor matrix.  Result register j = 5 u + b sits in row 8 (j / 4) + 4 h' + j % 4,
    // so row r belongs to lane half h' = (r / 4) % 2 and register j = 4 (r / 8) + r % 4.
    v4i afac[NM];
    {
        const uint32_t r = lane & 31u, hp = (r >> 2) & 1u, j = 4 * (r >> 3) + (r & 3u), u = j / 5, b = j - 5 * u;
        const int ta = min(t0 + (int)(hp * TL + u), n_dst - 1);  // a ragged last subset recomputes the last target
        const bool used = u < (uint32_t)TL;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const v4i* row = reinterpret_cast<const v4i*>(&P.afac[ta][b][2 * m + h][0]);
            afac[m] = used ? *row : v4i{0, 0, 0, 0};
        }
    }
    // per-lane constants of the targets this lane half receives: one 32-byte record each
    Mod mt[TL];
    int tgt[TL];
    uint32_t dst_limb[TL];
#pragma unroll
    for (int u = 0; u < TL; ++u) {
        tgt[u] = t0 + (int)h * TL + u;
        const BConvPlan::TargetRec rec = P.trec[min(tgt[u], n_dst - 1)];
        mt[u] = rec.m;
        dst_limb[u] = rec.limb;
    }
    // twiddles of all 2 TL targets -> LDS (requested now, written after the conversion, used after a barrier)
    constexpr int TW_PER_THREAD = (2 * TL * TW_WORDS + 255) / 256;
    double twv[TW_PER_THREAD];
#pragma unroll
    for (int i = 0; i < TW_PER_THREAD; ++i) {
        const uint32_t w = min(tid + 256u * i, 2u * TL * TW_WORDS - 1), ht = w / TW_WORDS, rem = w - ht * TW_WORDS;
        const int t = min(t0 + (int)ht, n_dst - 1);  // ht = half * TL + u, the order of the targets
        twv[i] = tw[(size_t)P.trec[t].mod_id * N + col_twiddle_index<LOG_R>(rem >> 4, rem & 15u)];
    }

    // Software pipeline over the 16 positions, fenced per position so that the schedule below is the one that runs
    // (left alone, the scheduler hoists every matrix instruction and spills): cut position k into bytes, re-request its
    // registers for position k + KB, issue its matrix instructions, then recombine position k - 1, whose results have had a
    // whole position's worth of instructions to arrive.
    double acc[TL][16];
    v16i sums[OVERLAP ? 2 : 1];
    auto recombine = [&](int k) {
        const v16i& s = sums[OVERLAP ? (k & 1) : 0];
#pragma unroll
        for (int u = 0; u < TL; ++u) {
            // sum_b 256^b S_b: the two low pairs fit 32-bit integers, the rest is exact in doubles
            const int lo = s[5 * u] + (s[5 * u + 1] << 8), mid = s[5 * u + 2] + (s[5 * u + 3] << 8);
            const double v = __builtin_fma((double)s[5 * u + 4], 4294967296.0, __builtin_fma((double)mid, 65536.0, (double)lo));
            acc[u][k] = reduce_lazy(v, mt[u]);
            // pin the recombined value here: otherwise the optimiser sinks these few instructions down to the butterflies
            // and keeps the 16 raw sums of every position alive instead (spilling them)
            asm volatile("" : "+v"(acc[u][k]));
        }
    };
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int kk = k % KB;
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            v4i bq = {0, 0, 0, 0};
            uint32_t top = 0;
#pragma unroll
            for (int e = 0; e < NPS; ++e) {
                const uint64_t bits = __builtin_bit_cast(uint64_t, yv[kk][m][e] + kDigitBias);
                bq[e] = (int)((uint32_t)bits ^ 0x80808080u);
                top |= ((uint32_t)(bits >> 32) & 0xFFu) << (8 * e);
                if (k + KB < 16)
                    yv[kk][m][e] = __builtin_bit_cast(
                        double, __builtin_amdgcn_raw_buffer_load_b64(ysrd, (int)voff[m][e], (int)((k + KB) * kStrideBytes), 0));
            }
            bq[3] = (int)top;
            s = __builtin_amdgcn_mfma_i32_32x32x32_i8(afac[m], bq, s, 0, 0, 0);
        }
        sums[OVERLAP ? (k & 1) : 0] = s;
        if (!OVERLAP) recombine(k);
        else if (k > 0) recombine(k - 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (OVERLAP) recombine(15);
#pragma unroll
    for (int i = 0; i < TW_PER_THREAD; ++i)
        if (tid + 256u * i < 2u * TL * TW_WORDS) lds_tw[tid + 256u * i] = twv[i];
    __syncthreads();

    // column half of the forward transform of each target, both lane halves at once (different moduli per half)
    double* lh = lds + h * HALF_WORDS;
#pragma unroll
    for (int u = 0; u < TL; ++u) {
        const double* ta = lds_tw + (h * TL + u) * TW_WORDS;
        radix16_fwd(acc[u], *reinterpret_cast<const double(*)[16]>(ta), mt[u]);
        if constexpr (E > 0) {
            if (u > 0) __syncthreads();  // the previous target's reads of the exchange buffer are done
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const uint32_t row = r0 + S * k;
                lh[row * TC + (row >> 4) * PADW + c] = acc[u][k];
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[u][k] = lh[(16 * r0 + k) * TC + r0 * PADW + c];
            radix16_fwd<4 - E>(acc[u], *reinterpret_cast<const double(*)[16]>(ta + 16 * (1 + r0)), mt[u]);
        }
        if (tgt[u] < n_dst) {
            uint64_t* dst = op + (uint64_t)dst_limb[u] * N;
#pragma unroll
            for (int k = 0; k < 16; ++k) store_f64(dst + col_row_grouped<LOG_R>(r0, k) * 256 + col, acc[u][k]);
        }
    }
}

// ---- row half of the forward transform of the raised limbs + inner product with the key (see ks_fused.hip) ----------
// One wavefront: four rows (group rg) of limb position pos of one batch item.  d_b / lifted_b / acc_b: that batch item's
// d [ell][N], raised digits [ndig][E][N] and accumulators [2][E][N].  lds_wave: 4 * kRowPitch doubles, lds_ta_wave: 64.
// accq_lo_b / accq_hi_b, packed_limbs: the first packed_limbs ciphertext limbs of the sums go to that batch item's packed
// [2][ell][N] accumulator instead of acc_b.
// WD / WK: word types of d and of the key (64-bit, or 32-bit for moduli below 2^32).
// PREFETCH (64-bit words only): loads are requested in the order x(0), key(0), x(1), key(1), ... and return in that order.
// While digit j is transformed, key(j) and x(j + 1) are in flight; every key slot is refilled with the next digit's as soon
// as its product is done, so key(j + 1) has the whole transform of digit j + 1 to arrive.
template <int LOG_R, typename WD, typename WK, bool PREFETCH = false>
__device__ __forceinline__ void task_rows_inner_product(const TwTables& tw, const TwTables& twi, const Mod* __restrict__ mods,
                                                        const DigitRanges& dg, uint32_t ell, uint32_t E, uint32_t L, uint32_t M,
                                                        const WD* __restrict__ d_b, const uint64_t* __restrict__ lifted_b,
                                                        const WK* __restrict__ evk, uint64_t* __restrict__ acc_b,
                                                        uint32_t* __restrict__ accq_lo_b, uint8_t* __restrict__ accq_hi_b,
                                                        uint32_t packed_limbs, uint32_t pos,
                                                        uint32_t rg, uint32_t lane, double* lds_wave, double* lds_ta_wave) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R;
    const uint32_t mid = pos < ell ? pos : L + (pos - ell);
    const Mod m = mods[mid];
    const uint32_t j0 = lane & 15, rr = lane >> 4, row = rg * 4 + rr;
    const uint32_t off = row * 256 + j0;
    double a0[16], a1[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) a0[k] = a1[k] = 0.0;
    // every digit's transform uses the same twiddles; the first-pass ones live in LDS to leave registers for a second
    // wavefront per SIMD
    double tb[16];
    row_twiddles_to_lds(lds_ta_wave + rr * 16, tw.W + (size_t)mid * N, R + row, j0);
    load_row_twiddles_b(tb, tw, mid, N, R + row, j0, m);
    __syncthreads();

    if constexpr (PREFETCH && sizeof(WD) == 8 && sizeof(WK) == 8) {
        const uint64_t* keys = reinterpret_cast<const uint64_t*>(evk) + (uint64_t)mid * N + off;
        const uint64_t comp = (uint64_t)M * N;
        auto source = [&](uint32_t j) {
            const bool own = pos >= dg.lo[j] && pos < dg.hi[j];  // uniform
            return own ? reinterpret_cast<const uint64_t*>(d_b) + (uint64_t)pos * N + off : lifted_b + ((uint64_t)j * E + pos) * N + off;
        };
        uint64_t xn[16], kc0[16], kc1[16];
        {
            const uint64_t* src = source(0);
#pragma unroll
            for (int k = 0; k < 16; ++k) xn[k] = src[16 * k];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                kc0[k] = keys[16 * k];
                kc1[k] = keys[comp + 16 * k];
            }
        }
        auto digit = [&](uint32_t j, auto next) {
            constexpr bool NEXT = decltype(next)::value;
            const bool own = pos >= dg.lo[j] && pos < dg.hi[j];  // uniform
            double x[16];
            if (own) {
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = u64_to_f64(xn[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = __longlong_as_double((long long)xn[k]);
            }
            const uint64_t* kp = keys + (uint64_t)(j + 1) * 2 * comp;
            if constexpr (NEXT) {
                const uint64_t* src = source(j + 1);
#pragma unroll
                for (int k = 0; k < 16; ++k) xn[k] = src[16 * k];
            }
            if (!own) row_fwd_core_lds(x, lds_ta_wave + rr * 16, tb, j0, lds_wave + rr * kRowPitch, m);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                a0[k] += mulmod_lazy(x[k], u64_to_f64(kc0[k]), m);
                a1[k] += mulmod_lazy(x[k], u64_to_f64(kc1[k]), m);
                if constexpr (NEXT) {
                    kc0[k] = kp[16 * k];
                    kc1[k] = kp[comp + 16 * k];
                }
            }
        };
#pragma unroll 1
        for (uint32_t j = 0; j + 1 < dg.ndig; ++j) digit(j, std::true_type{});
        digit(dg.ndig - 1, std::false_type{});
    } else {
#pragma unroll 1
    for (uint32_t j = 0; j < dg.ndig; ++j) {
        const bool own = pos >= dg.lo[j] && pos < dg.hi[j];  // uniform
        const WK* key0 = evk + ((uint64_t)(j * 2 + 0) * M + mid) * N + off;
        const WK* key1 = evk + ((uint64_t)(j * 2 + 1) * M + mid) * N + off;
        // issue every load of this digit up front (the key slots are independent of the transform below)
        double x[16], k0[16], k1[16];
        if constexpr (sizeof(WD) == 8 && sizeof(WK) == 8) {
            const uint64_t* src = own ? reinterpret_cast<const uint64_t*>(d_b) + (uint64_t)pos * N + off
                                      : lifted_b + ((uint64_t)j * E + pos) * N + off;
            uint64_t raw[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) raw[k] = src[16 * k];
#pragma unroll
            for (int k = 0; k < 16; ++k) k0[k] = word_to_f64<WK>(key0[16 * k]);
#pragma unroll
            for (int k = 0; k < 16; ++k) k1[k] = word_to_f64<WK>(key1[16 * k]);
            if (own) {
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = u64_to_f64(raw[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = __longlong_as_double((long long)raw[k]);
                row_fwd_core_lds(x, lds_ta_wave + rr * 16, tb, j0, lds_wave + rr * kRowPitch, m);
            }
        } else {
            // the digit's own limbs come in boundary words, the raised ones as raw doubles: two load shapes, so the
            // (uniform) choice is a branch; the key slots are requested before it and everything is awaited after it
            WK kr0[16], kr1[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) kr0[k] = key0[16 * k];
#pragma unroll
            for (int k = 0; k < 16; ++k) kr1[k] = key1[16 * k];
            if (own) {
                const WD* src = d_b + (uint64_t)pos * N + off;
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = word_to_f64<WD>(src[16 * k]);
            } else {
                const uint64_t* src = lifted_b + ((uint64_t)j * E + pos) * N + off;
#pragma unroll
                for (int k = 0; k < 16; ++k) x[k] = load_f64(src + 16 * k);
                row_fwd_core_lds(x, lds_ta_wave + rr * 16, tb, j0, lds_wave + rr * kRowPitch, m);
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) k0[k] = word_to_f64<WK>(kr0[k]);
#pragma unroll
            for (int k = 0; k < 16; ++k) k1[k] = word_to_f64<WK>(kr1[k]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            a0[k] += mulmod_lazy(x[k], k0[k], m);
            a1[k] += mulmod_lazy(x[k], k1[k], m);
        }
    }
    }
    uint64_t* o0 = acc_b + ((uint64_t)0 * E + pos) * N + off;
    uint64_t* o1 = acc_b + ((uint64_t)1 * E + pos) * N + off;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        a0[k] = reduce_lazy(a0[k], m);
        a1[k] = reduce_lazy(a1[k], m);
    }
    if (pos < packed_limbs) {
        // uniform: ciphertext limbs are kept in evaluation domain for the final subtract-and-scale, which is their only
        // reader: they go out packed, bits 0..31 as a 32-bit word and the bits above as a byte, [2][ell][N] per batch item
        const uint64_t e0 = (uint64_t)pos * N + off, e1 = e0 + (uint64_t)ell * N;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint64_t u0 = f64_to_u64(canon(a0[k], m)), u1 = f64_to_u64(canon(a1[k], m));
            accq_lo_b[e0 + 16 * k] = (uint32_t)u0;
            accq_lo_b[e1 + 16 * k] = (uint32_t)u1;
            accq_hi_b[e0 + 16 * k] = (uint8_t)(u0 >> 32);
            accq_hi_b[e1 + 16 * k] = (uint8_t)(u1 >> 32);
        }
    } else if (pos < ell) {  // uniform: a ciphertext limb that another kernel reads as a 64-bit word
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            o0[16 * k] = f64_to_u64(canon(a0[k], m));
            o1[16 * k] = f64_to_u64(canon(a1[k], m));
        }
    } else {
        // Special limbs go straight into ModDown: the row half of their inverse transform works on the very
        // rows this wavefront holds, so it is done here and raw doubles are handed to the column half.
        PassTwiddles ti;
        load_row_twiddles(ti, twi, mid, N, R + row, j0, m);
        row_inv_core(a0, ti, j0, lds_wave + rr * kRowPitch, m);
        row_inv_core(a1, ti, j0, lds_wave + rr * kRowPitch, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            store_f64(o0 + 16 * k, a0[k]);
            store_f64(o1 + 16 * k, a1[k]);
        }
    }
}

// ---- row half of the forward transform of the converted limbs + (acc - conv) * mul (+ addend) ------------------------
// One wavefront: four rows (group rg) of limb i.  src / ap / op: that limb of conv, of the accumulator and of the output;
// adp: that limb of the addend (ADDEND != 0).  ADDEND: 0 = none, 1 = added as it is, 2 = multiplied by admul first.
// ACCP: the accumulator limb is packed, bits 0..31 as 32-bit words at ap and the bits above as bytes at ap_hi.
// ADF: format of the addend limb: 0 = 64-bit words, 1 = packed like the accumulator (adp, adp_hi; read in place only),
// 2 = 32-bit words.
template <int LOG_R, bool GATHER, int ADDEND, typename W, bool ACCP = false, int ADF = 0>
__device__ __forceinline__ void task_rows_finish(const TwTables& tw, Mod m, uint32_t mod_id, double mul, double admul,
                                                 const uint64_t* __restrict__ src, const void* __restrict__ ap,
                                                 const uint8_t* __restrict__ ap_hi, W* __restrict__ op,
                                                 const void* __restrict__ adp, const uint8_t* __restrict__ adp_hi,
                                                 uint32_t galois, uint32_t rg, uint32_t lane, double* lds_wave) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, LOGN = LOG_R + 8;
    const uint32_t j0 = lane & 15, rr = lane >> 4, row = rg * 4 + rr;
    const uint32_t off = row * 256 + j0;
    // issue every load up front: the accumulator (and addend) slots do not depend on the transform
    double w[16], a[16], ad[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) w[k] = load_f64(src + off + 16 * k);
    if constexpr (ACCP) {
        uint32_t alo[16], ahi[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) alo[k] = static_cast<const uint32_t*>(ap)[off + 16 * k];
#pragma unroll
        for (int k = 0; k < 16; ++k) ahi[k] = ap_hi[off + 16 * k];
#pragma unroll
        for (int k = 0; k < 16; ++k) a[k] = u64_to_f64((uint64_t)ahi[k] << 32 | alo[k]);
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) a[k] = u64_to_f64(static_cast<const uint64_t*>(ap)[off + 16 * k]);
    }
    if constexpr (ADDEND != 0 && ADF == 1) {
        static_assert(!GATHER || ADF != 1, "a packed addend is read in place");
        uint32_t dlo[16], dhi[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) dlo[k] = static_cast<const uint32_t*>(adp)[off + 16 * k];
#pragma unroll
        for (int k = 0; k < 16; ++k) dhi[k] = adp_hi[off + 16 * k];
#pragma unroll
        for (int k = 0; k < 16; ++k) ad[k] = u64_to_f64((uint64_t)dhi[k] << 32 | dlo[k]);
    } else if constexpr (ADDEND != 0) {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t n = off + 16 * k;
            const uint32_t sn = GATHER ? galois_source_slot(n, galois, LOGN) : n;
            if constexpr (ADF == 2) ad[k] = (double)static_cast<const uint32_t*>(adp)[sn];
            else ad[k] = u64_to_f64(static_cast<const uint64_t*>(adp)[sn]);
        }
    }
    PassTwiddles t;
    load_row_twiddles(t, tw, mod_id, N, R + row, j0, m);
    row_fwd_core(w, t, j0, lds_wave + rr * kRowPitch, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        double r = mulmod_lazy(a[k] - w[k], mul, m);
        if constexpr (ADDEND == 1) r = reduce_lazy(r + ad[k], m);
        if constexpr (ADDEND == 2) r = reduce_lazy(r + mulmod_lazy(ad[k], admul, m), m);
        op[off + 16 * k] = f64_to_word<W>(canon(r, m));
    }
}

}  // namespace ks
