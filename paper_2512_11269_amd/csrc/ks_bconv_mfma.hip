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
#include "ks_tasks.hpp"

namespace ks {

// Workgroups per compute unit the register allocation must leave room for: without a bound the scheduler hoists the
// matrix instructions of all 16 positions (256 result registers) and the kernel drops to one wavefront per SIMD.
constexpr int mfma_min_blocks(int tl) { return tl == 1 ? 4 : 2; }

template <int LOG_R, int TL, int NM, int NPS>
__global__ __launch_bounds__(256, mfma_min_blocks(TL)) void bconv_mfma_ntt_cols(const double* __restrict__ tw, const BConvPlan* __restrict__ plans,
                                                           LaunchMeta meta, const uint64_t* __restrict__ y, uint64_t y_ps,
                                                           uint64_t* __restrict__ out, uint64_t out_ps, uint32_t n_subsets) {
    using Shape = MfmaConvShape<LOG_R, TL>;
    __shared__ double lds[Shape::LDS_WORDS];
    __shared__ double lds_tw[Shape::LDS_TW_WORDS];
    const uint32_t plan_id = blockIdx.y / n_subsets, subset = blockIdx.y - plan_id * n_subsets;
    const PlanMeta& PM = meta.plan[plan_id];  // kernel arguments: scalar loads, nothing else to wait for
    const int t0 = (int)subset * 2 * TL;
    if (t0 >= (int)PM.n_dst) return;  // uniform for the whole workgroup
    task_bconv_mfma_cols<LOG_R, TL, NM, NPS>(tw, plans[plan_id], PM, y + (uint64_t)blockIdx.z * y_ps, y_ps * 8,
                                             out + (uint64_t)blockIdx.z * out_ps, blockIdx.x, t0, threadIdx.x, lds, lds_tw);
}

// Targets per lane half: one gives the most workgroups, three shares the byte-cutting of the sources among the most
// targets (and keeps the stores of one target under the butterflies of the next).
void launch_bconv_mfma_ntt_cols(const ks_ctx* c, const PlanSet& plans, const uint64_t* y, uint64_t y_ps, uint64_t* out,
                                uint64_t out_ps, uint32_t n_polys, int tl, hipStream_t s) {
    const uint32_t n_src = plans.shape_src, n_plans = plans.n_plans, max_targets = plans.max_targets;
    const BConvPlan* d_plans = plans.d_plans;
    const uint32_t nm = (n_src + 5) / 6, nps = (n_src + 2 * nm - 1) / (2 * nm);
    const uint32_t tiles = c->N / 2048;
    tl = (c->logN != 12 && c->logN != 16) || tl < 2 ? 1 : 3;  // built shapes: one or three targets per lane half
    const uint32_t n_subsets = (max_targets + 2 * tl - 1) / (2 * tl);
    const dim3 grid(tiles, n_plans * n_subsets, n_polys), block(256);
#define KS_LAUNCH_MFMA(LOGR, TLV, NMV, NPSV)                                                                                        \
    hipLaunchKernelGGL((bconv_mfma_ntt_cols<LOGR, TLV, NMV, NPSV>), grid, block, 0, s, c->d_tw_fwd, d_plans, plans.meta, y, y_ps, \
                       out, out_ps, n_subsets)
#define KS_MFMA_SHAPE(LOGR, TLV)                                      \
    if (nm == 1 && nps == 1) KS_LAUNCH_MFMA(LOGR, TLV, 1, 1);         \
    else if (nm == 1 && nps == 2) KS_LAUNCH_MFMA(LOGR, TLV, 1, 2);    \
    else if (nm == 1) KS_LAUNCH_MFMA(LOGR, TLV, 1, 3);                \
    else if (nm == 2 && nps == 2) KS_LAUNCH_MFMA(LOGR, TLV, 2, 2);    \
    else if (nm == 2) KS_LAUNCH_MFMA(LOGR, TLV, 2, 3);                \
    else KS_LAUNCH_MFMA(LOGR, TLV, 3, 3)
    // every shape for the benchmarked ring degree and for the smallest one (which the parity sweeps run on); the degrees
    // in between take one target per lane half
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
