// Base conversion on the matrix cores (int8 MFMA), fused with the column half of the forward transform of every target
// limb (Kernel Code Generation: "Base Conversion" kernel class; the tensor-core formulations in the paper's Related Work).
//
// The conversion sum  out_t = sum_i y_i (D / s_i)  (mod t)  is a contraction over the sources i with one modulus per
// output column, so it cannot run on the matrix cores as it stands.  Cut into bytes it can: y_i = sum_a d_{i,a} 256^a
// with five signed digits d (|d| <= 128), and for every digit position the factor [(D / s_i) 256^a]_t, centred, is cut
// the same way into digits e_{t,i,a,b}.  Then
//     y_i (D / s_i) = sum_b 256^b  S_b   (mod t),     S_b = sum_{i,a} d_{i,a} e_{t,i,a,b},
// and the five S_b of a target are dot products of length 5 n_src over small integers: one row of an int8 matrix
// product with exact 32-bit accumulation (|S_b| <= 16 * 5 * 2^14).  The recombined value is below 2^49 in magnitude,
// exact in a double, and one Barrett step makes it a lazy residue modulo t.
//
// v_mfma_i32_32x32x32_i8: every lane supplies 16 bytes of A (row = lane % 32) and 16 bytes of B (column = lane % 32) for
// the 16 contraction indices of its half (lane / 32); result register j of a lane holds row 8 (j / 4) + 4 (lane / 32) + j % 4
// of its column.  Here a COLUMN IS A COEFFICIENT POSITION, so the B operand of a lane is made of the bytes of that lane's
// own source residues: no data crosses lanes on the way in.  The two lanes that share a column (l and l + 32) read
// different sources and receive different targets: rows are ordered so that result registers 5 u + b of a lane are the
// five digit planes b of its u-th target.  A workgroup owns a tile of 2048 positions and 2 TL targets (TL per lane half):
// thread (pair p = 32 wave + lane % 32, half h) walks the 16 positions (row r0 + 16 k, column c) of pair p, exactly the
// points the column butterflies need in its registers afterwards.
#include "ks_internal.hpp"
#include "ks_tiles.hpp"

namespace ks {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Adding 2^52 + 0x80808080 to a canonical residue y < 2^36 (held as a double) leaves y + 0x80808080 in the mantissa:
// its low four bytes, each with the top bit flipped, are the signed digits d_0..d_3 (digit = byte - 128), and bits
// 32..39 are the non-negative digit d_4 <= 16.
constexpr double kDigitBias = 4503599627370496.0 + 2155905152.0;

#ifdef KS_EXP_TRACE
// phase timestamps of every wavefront (tuning builds only)
__device__ unsigned long long g_trace[1 << 15][8];
#define KS_TRACE(phase)                                                                                               \
    do {                                                                                                              \
        if ((threadIdx.x & 63u) == 0) {                                                                               \
            const uint32_t w_ = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + (threadIdx.x >> 6); \
            if (w_ < (1u << 15)) g_trace[w_][phase] = __builtin_readcyclecounter();                                   \
        }                                                                                                             \
    } while (0)
#else
#define KS_TRACE(phase)
#endif

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

// Workgroups per compute unit the register allocation must leave room for: without a bound the scheduler hoists the
// matrix instructions of all 16 positions (256 result registers) and the kernel drops to one wavefront per SIMD.
constexpr int mfma_min_blocks(int tl) { return tl == 1 ? 4 : 2; }

template <int LOG_R, int TL, int NM, int NPS>
__global__ __launch_bounds__(256, mfma_min_blocks(TL)) void bconv_mfma_ntt_cols(const double* __restrict__ tw, const BConvPlan* __restrict__ plans,
                                                           LaunchMeta meta, const uint64_t* __restrict__ y, uint64_t y_ps,
                                                           uint64_t* __restrict__ out, uint64_t out_ps, uint32_t n_subsets) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, TC = 2048u >> LOG_R;  // tile: TC columns x R rows
    constexpr int E = LOG_R - 4, S = 1 << E;
    // exchange buffer of the column butterflies, one region per lane half; rows are padded so that the 16-row groups the
    // second pass reads start in different banks
    constexpr uint32_t PADW = TC <= 16 ? TC : 0, HALF_WORDS = R * TC + (R / 16) * PADW;
    constexpr uint32_t TW_WORDS = (1 + S) * 16;  // per (half, target)
    __shared__ double lds[LOG_R > 4 ? 2 * HALF_WORDS : 1];
    __shared__ double lds_tw[2 * TL * TW_WORDS];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, h = lane >> 5, p = (tid >> 6) * 32u + (lane & 31u);
    const uint32_t c = p & (TC - 1), r0 = p / TC, col = blockIdx.x * TC + c;
    KS_TRACE(0);
    const uint32_t plan_id = blockIdx.y / n_subsets, subset = blockIdx.y - plan_id * n_subsets;
    const PlanMeta& PM = meta.plan[plan_id];  // kernel arguments: scalar loads, nothing else to wait for
    const BConvPlan& P = plans[plan_id];
    const int n_dst = (int)PM.n_dst;
    const int t0 = (int)subset * 2 * TL;
    if (t0 >= n_dst) return;  // uniform for the whole workgroup
    const uint64_t* yp = y + (uint64_t)blockIdx.z * y_ps;
    uint64_t* op = out + (uint64_t)blockIdx.z * out_ps;

    // B operand: the sources of this lane's slots, read through a buffer descriptor (per-lane offset = position + limb).
    // The first half of the positions is requested before anything else.
    const BufferRsrc ysrd = make_buffer_rsrc(yp, y_ps * 8);
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
    KS_TRACE(1);

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
    KS_TRACE(2);

    // column half of the forward transform of each target, both lane halves at once (different moduli per half)
    double* lh = lds + h * HALF_WORDS;
#pragma unroll
    for (int u = 0; u < TL; ++u) {
        const double* ta = lds_tw + (h * TL + u) * TW_WORDS;
        radix16_fwd(acc[u], *reinterpret_cast<const double(*)[16]>(ta), mt[u]);
        if (u == 0) KS_TRACE(3);
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
        if (u == 0) KS_TRACE(4);
        if (tgt[u] < n_dst) {
            uint64_t* dst = op + (uint64_t)dst_limb[u] * N;
#pragma unroll
            for (int k = 0; k < 16; ++k) store_f64(dst + col_row_grouped<LOG_R>(r0, k) * 256 + col, acc[u][k]);
        }
    }
    KS_TRACE(5);
#ifdef KS_EXP_TRACE
    __builtin_amdgcn_s_waitcnt(0);
    KS_TRACE(6);
#endif
}

#ifdef KS_EXP_TRACE
extern "C" int ks_debug_trace_read(unsigned long long* host, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), bytes);
}
#endif

// Targets per lane half: one gives the most workgroups (single-ciphertext launches are latency-bound and want the chip
// full of short workgroups), three shares the byte-cutting of the sources among the most targets.
void launch_bconv_mfma_ntt_cols(const ks_ctx* c, const PlanSet& plans, const uint64_t* y, uint64_t y_ps, uint64_t* out,
                                uint64_t out_ps, uint32_t n_polys, int tl, hipStream_t s) {
    const uint32_t n_src = plans.shape_src, n_plans = plans.n_plans, max_targets = plans.max_targets;
    const BConvPlan* d_plans = plans.d_plans;
    const uint32_t nm = (n_src + 5) / 6, nps = (n_src + 2 * nm - 1) / (2 * nm);
    const uint32_t tiles = c->N / 2048;
    tl = (c->logN != 12 && c->logN != 16) || tl < 2 ? 1 : 3;  // built shapes: one or three targets per lane half
    const uint32_t n_subsets = (max_targets + 2 * tl - 1) / (2 * tl);
    const dim3 grid(tiles, n_plans * n_subsets, n_polys), block(256);
#define KS_LAUNCH_MFMA(LOGR, TLV, NMV, NPSV)                                                                                    \
    hipLaunchKernelGGL((bconv_mfma_ntt_cols<LOGR, TLV, NMV, NPSV>), grid, block, 0, s, c->d_tw_fwd, d_plans, plans.meta, y, y_ps, \
                       out, out_ps, n_subsets)
#define KS_MFMA_SHAPE(LOGR, TLV)                                      \
    if (nm == 1 && nps == 1) KS_LAUNCH_MFMA(LOGR, TLV, 1, 1);         \
    else if (nm == 1 && nps == 2) KS_LAUNCH_MFMA(LOGR, TLV, 1, 2);    \
    else if (nm == 1) KS_LAUNCH_MFMA(LOGR, TLV, 1, 3);                \
    else if (nm == 2 && nps == 2) KS_LAUNCH_MFMA(LOGR, TLV, 2, 2);    \
    else if (nm == 2) KS_LAUNCH_MFMA(LOGR, TLV, 2, 3);                \
    else KS_LAUNCH_MFMA(LOGR, TLV, 3, 3)
    // every TL for the benchmarked ring degree and for the smallest one (which the parity sweeps run on); the degrees
    // in between take TL = 1
#define KS_LAUNCH_TL(LOGR)                   \
    if (tl == 1) { KS_MFMA_SHAPE(LOGR, 1); } \
    else { KS_MFMA_SHAPE(LOGR, 3); }
    switch (c->logN) {
        case 12: KS_LAUNCH_TL(4); break;
        case 13: KS_MFMA_SHAPE(5, 1); break;
        case 14: KS_MFMA_SHAPE(6, 1); break;
        case 15: KS_MFMA_SHAPE(7, 1); break;
        default: KS_LAUNCH_TL(8); break;
    }
#undef KS_LAUNCH_TL
#undef KS_MFMA_SHAPE
#undef KS_LAUNCH_MFMA
}

// ------------------------------------------------------------------------------------------------
// Standalone conversion on the matrix cores (the `bconv` entry point's second kernel): canonical residues in, canonical
// residues out, no transform.  A wavefront owns 32 consecutive positions: lane (position l % 32, half l / 32) scales
// its slots' source residues to y_i = [x_i (D / s_i)^-1]_{s_i}, cuts them into bytes once, and then walks the targets six
// at a time (three per lane half), writing 256-byte segments per target.
// ------------------------------------------------------------------------------------------------
template <int NM, int NPS>
__global__ __launch_bounds__(256) void bconv_mfma_kernel(const BConvPlan* __restrict__ plans, LaunchMeta meta,
                                                         const uint64_t* __restrict__ in, uint64_t in_ps,
                                                         uint64_t* __restrict__ out, uint64_t out_ps, uint32_t N) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u, h = lane >> 5;
    const uint32_t n = (blockIdx.x * 4 + (tid >> 6)) * 32 + (lane & 31u);  // N is a multiple of 128
    const BConvPlan& P = plans[blockIdx.y];
    const int n_dst = (int)meta.plan[blockIdx.y].n_dst, n_src = (int)P.n_src;
    const uint64_t* ip = in + (uint64_t)blockIdx.z * in_ps + n;
    uint64_t* op = out + (uint64_t)blockIdx.z * out_ps + n;
    v4i bq[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        bq[m] = v4i{0, 0, 0, 0};
        uint32_t top = 0;
#pragma unroll
        for (int e = 0; e < NPS; ++e) {
            const int i = min((int)((2 * m + h) * NPS + e), n_src - 1);  // slots past the last source repeat it against zero factors
            const Mod mi = P.src_mod[i];
            const double x = u64_to_f64(ip[(uint64_t)P.src_limb[i] * N]);
            const double yi = canon(mulmod_lazy(x, P.src_inv[i], mi), mi);
            const uint64_t bits = __builtin_bit_cast(uint64_t, yi + kDigitBias);
            bq[m][e] = (int)((uint32_t)bits ^ 0x80808080u);
            top |= ((uint32_t)(bits >> 32) & 0xFFu) << (8 * e);
        }
        bq[m][3] = (int)top;
    }
    const uint32_t r = lane & 31u, hp = (r >> 2) & 1u, j = 4 * (r >> 3) + (r & 3u), ua = j / 5, b = j - 5 * ua;
#pragma unroll 1
    for (int t0 = 0; t0 < n_dst; t0 += 6) {
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const int ta = min(t0 + (int)(hp * 3 + ua), n_dst - 1);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const v4i afac = ua < 3 ? *reinterpret_cast<const v4i*>(&P.afac[ta][b][2 * m + h][0]) : v4i{0, 0, 0, 0};
            s = __builtin_amdgcn_mfma_i32_32x32x32_i8(afac, bq[m], s, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int t = t0 + (int)h * 3 + u;
            if (t < n_dst) {
                const BConvPlan::TargetRec rec = P.trec[t];
                const int lo = s[5 * u] + (s[5 * u + 1] << 8), mid = s[5 * u + 2] + (s[5 * u + 3] << 8);
                const double v = __builtin_fma((double)s[5 * u + 4], 4294967296.0, __builtin_fma((double)mid, 65536.0, (double)lo));
                op[(uint64_t)rec.limb * N] = f64_to_u64(canon(reduce_lazy(v, rec.m), rec.m));
            }
        }
    }
}

void launch_bconv_mfma(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const uint64_t* in, uint64_t in_ps,
                       uint64_t* out, uint64_t out_ps, uint32_t n_polys, hipStream_t s) {
    if (n_polys == 0 || plans.n_plans == 0) return;
    const uint32_t n_src = plans.shape_src, nm = (n_src + 5) / 6, nps = (n_src + 2 * nm - 1) / (2 * nm);
    const dim3 grid(c->N / 128, plans.n_plans, n_polys), block(256);
    ProfScope ps("bconv_mfma", (double)limbs_moved_per_poly * n_polys * c->N * 8.0, s);
#define KS_LAUNCH_BM(NMV, NPSV) \
    hipLaunchKernelGGL((bconv_mfma_kernel<NMV, NPSV>), grid, block, 0, s, plans.d_plans, plans.meta, in, in_ps, out, out_ps, c->N)
    if (nm == 1 && nps == 1) KS_LAUNCH_BM(1, 1);
    else if (nm == 1 && nps == 2) KS_LAUNCH_BM(1, 2);
    else if (nm == 1) KS_LAUNCH_BM(1, 3);
    else if (nm == 2 && nps == 2) KS_LAUNCH_BM(2, 2);
    else if (nm == 2) KS_LAUNCH_BM(2, 3);
    else KS_LAUNCH_BM(3, 3);
#undef KS_LAUNCH_BM
}

}  // namespace ks
