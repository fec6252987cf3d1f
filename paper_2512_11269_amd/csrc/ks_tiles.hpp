// Tile-level pieces of the two-phase transform, shared by the plain NTT kernels and the fused ones.
//
// A limb is an R x 256 matrix (R = N / 256 = 16 .. 256).  "Row" pieces work on contiguous 256-point rows, one
// wavefront owning four rows (16 lanes per row, 16 points per lane); "column" pieces work on a tile of 4096 / R
// columns x R rows (16 x 256 for N = 2^16) owned by a 256-thread workgroup.  Twiddles come from the per-modulus heap-ordered
// table W[k] = psi^brv(k): the forward stage with 2^s blocks uses W[2^s + block].
#pragma once
#include "ks_device.hpp"

namespace ks {

// Digit partition handed to kernels by value.
struct DigitRanges {
    uint32_t ndig;
    uint32_t lo[8], hi[8];
};

// Slot permutation of sigma_g (X -> X^g) on a bit-reversed evaluation vector: slot n holds the point
// psi^(2 brv(n) + 1); sigma_g(a) evaluated there is a evaluated at that point raised to g.
__device__ __forceinline__ uint32_t galois_source_slot(uint32_t n, uint32_t g, uint32_t logN) {
    const uint32_t e = (g * (2u * (__brev(n) >> (32 - logN)) + 1u)) & ((2u << logN) - 1u);
    return __brev((e - 1u) >> 1) >> (32 - logN);
}

constexpr int kRowPitch = 272;  // 256 points + 1 pad per 16: the transposed LDS accesses hit distinct banks

__device__ __forceinline__ double load_f64(const uint64_t* p) { return *reinterpret_cast<const double*>(p); }
__device__ __forceinline__ void store_f64(uint64_t* p, double v) { *reinterpret_cast<double*>(p) = v; }

// Twiddles of the two register passes of a tile core, loaded ahead of the butterflies.
struct PassTwiddles {
    double a[16], b[16];
};
// One direction's twiddle tables (device pointers, every table indexed [modulus id][...]):
//   W    [N]     W[k] = psi^brv(k) (or psi^-brv(k)), heap order
//   trow [N/16]  trow[i] = W[8 (N/16 + i)] = psi^(1 + 2 brv(i)): the generator of the last register pass of row-pass lane i
//   w16  [8]     w16[e] = omega^e, omega = psi^(N/8) a primitive 16th root of unity
struct TwTables {
    const double* W;
    const double* trow;
    const double* w16;
};

// rows: node = R + row; lane j0 owns points 16 j0 .. 16 j0 + 15 in the second pass.
// The second pass needs the 15 table entries below heap node n = 16 node + j0 -- one twiddle per point of the row,
// as much data as the row itself.  They factor as W[n 2^u + g] = T^(2^(3-u)) * omega^(2^(3-u) brv_u(g)) with
// T = W[8 n], so one load, three squarings and eleven products replace fifteen loads (row kernels are
// bandwidth-bound and have arithmetic to spare).
__device__ __forceinline__ void load_row_twiddles(PassTwiddles& t, const TwTables& tb, uint32_t mod_id, uint32_t N, uint32_t node,
                                                  uint32_t j0, Mod m) {
    load_twiddles16(t.a, tb.W + (size_t)mod_id * N, node);
    const double* w = tb.w16 + mod_id * 8;
    const double T1 = tb.trow[(size_t)mod_id * (N / 16) + (node * 16 + j0 - N / 16)];
    const double T2 = mulmod_lazy(T1, T1, m), T4 = mulmod_lazy(T2, T2, m), T8 = mulmod_lazy(T4, T4, m);
    t.b[0] = 0.0;
    t.b[1] = T8;
    t.b[2] = T4;  t.b[3] = mulmod_lazy(T4, w[4], m);
    t.b[4] = T2;  t.b[5] = mulmod_lazy(T2, w[4], m);  t.b[6] = mulmod_lazy(T2, w[2], m);  t.b[7] = mulmod_lazy(T2, w[6], m);
    t.b[8] = T1;  t.b[9] = mulmod_lazy(T1, w[4], m);  t.b[10] = mulmod_lazy(T1, w[2], m); t.b[11] = mulmod_lazy(T1, w[6], m);
    t.b[12] = mulmod_lazy(T1, w[1], m);  t.b[13] = mulmod_lazy(T1, w[5], m);
    t.b[14] = mulmod_lazy(T1, w[3], m);  t.b[15] = mulmod_lazy(T1, w[7], m);
}
// The same with the first-pass twiddles left out (for kernels that keep them in LDS, see row_twiddles_to_lds).
__device__ __forceinline__ void load_row_twiddles_b(double (&tb)[16], const TwTables& tbl, uint32_t mod_id, uint32_t N, uint32_t node,
                                                    uint32_t j0, Mod m) {
    const double* w = tbl.w16 + mod_id * 8;
    const double T1 = tbl.trow[(size_t)mod_id * (N / 16) + (node * 16 + j0 - N / 16)];
    const double T2 = mulmod_lazy(T1, T1, m), T4 = mulmod_lazy(T2, T2, m), T8 = mulmod_lazy(T4, T4, m);
    tb[0] = 0.0;
    tb[1] = T8;
    tb[2] = T4;  tb[3] = mulmod_lazy(T4, w[4], m);
    tb[4] = T2;  tb[5] = mulmod_lazy(T2, w[4], m);  tb[6] = mulmod_lazy(T2, w[2], m);  tb[7] = mulmod_lazy(T2, w[6], m);
    tb[8] = T1;  tb[9] = mulmod_lazy(T1, w[4], m);  tb[10] = mulmod_lazy(T1, w[2], m); tb[11] = mulmod_lazy(T1, w[6], m);
    tb[12] = mulmod_lazy(T1, w[1], m);  tb[13] = mulmod_lazy(T1, w[5], m);
    tb[14] = mulmod_lazy(T1, w[3], m);  tb[15] = mulmod_lazy(T1, w[7], m);
}
// First-pass twiddles of a row (the 15 table entries below heap node `node`, the same for the row's 16 lanes) placed in
// 16 doubles of LDS: lane j0 fetches entry j0.  Frees 30 registers per lane where a kernel is short of them; the
// butterflies then read them as LDS broadcasts.  The caller synchronises before use.
__device__ __forceinline__ void row_twiddles_to_lds(double* ta_row, const double* __restrict__ W, uint32_t node, uint32_t j0) {
    const uint32_t u = 31u - __clz(j0 | 1u), g = j0 - (1u << u);
    ta_row[j0] = j0 ? W[(node << u) + g] : 0.0;
}

// Columns (R = 2^LOG_R rows, 4 <= LOG_R <= 8): the first register pass runs global stages 0..3 with the sub-tree below
// heap node 1; the second one the remaining E = LOG_R - 4 stages on 16 consecutive rows 16 r0 + k, as the last E local
// stages of a 16-point pass: local stage ul = 4 - E + u is global stage 4 + u, whose block of row 16 r0 + k is
// r0 2^ul + (k >> (4 - ul)), so its table entry (1 << ul) + g holds W[2^(E + ul) + r0 2^ul + g].  For E = 4 that is
// the sub-tree below node 16 + r0.
template <int LOG_R>
__device__ __forceinline__ void load_col_twiddles(PassTwiddles& t, const double* __restrict__ W, uint32_t r0) {
    constexpr int E = LOG_R - 4;
    load_twiddles16(t.a, W, 1);
    if constexpr (E > 0) {
#pragma unroll
        for (int ul = 4 - E; ul < 4; ++ul)
#pragma unroll
            for (int g = 0; g < (1 << ul); ++g) t.b[(1 << ul) + g] = W[(1u << (E + ul)) + (r0 << ul) + g];
    }
}

// Last 8 forward stages of one row.  in: v[k] = point j0 + 16 k of the row, lazy with |v| <= 8 p.
// out: v[k] = transformed point j0 + 16 k, lazy with |v| <= |in| + 4.1 p.
// lrow: this row's kRowPitch doubles of LDS, shared by the row's 16 lanes (all in one wavefront).
__device__ __forceinline__ void row_fwd_core(double (&v)[16], const PassTwiddles& t, uint32_t j0, double* lrow, Mod m) {
    radix16_fwd(v, t.a, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_fwd(v, t.b, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[17 * j0 + k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[j0 + 17 * k];
}

// The same without the last exchange: out v[k] = point 16 j0 + k (sixteen consecutive points per thread).
__device__ __forceinline__ void row_fwd_core_consecutive(double (&v)[16], const PassTwiddles& t, uint32_t j0, double* lrow, Mod m) {
    radix16_fwd(v, t.a, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_fwd(v, t.b, m);
}

// The same with the first-pass twiddles read from LDS (ta: 16 doubles of this row) and the second-pass ones in registers.
__device__ __forceinline__ void row_fwd_core_lds(double (&v)[16], const double* ta, const double (&tb)[16], uint32_t j0, double* lrow,
                                                 Mod m) {
    radix16_fwd(v, *reinterpret_cast<const double(*)[16]>(ta), m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_fwd(v, tb, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[17 * j0 + k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[j0 + 17 * k];
}

// First 8 inverse stages of one row (t built from the inverse table).  in: v[k] = point j0 + 16 k, |v| <= p.
// out: same layout, |v| <= 0.51 p.
__device__ __forceinline__ void row_inv_core(double (&v)[16], const PassTwiddles& t, uint32_t j0, double* lrow, Mod m) {
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_inv(v, t.b, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[17 * j0 + k] = reduce_lazy(v[k], m);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[j0 + 17 * k];
    radix16_inv(v, t.a, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = reduce_lazy(v[k], m);
}

// First log2(R) forward stages on a column tile of TC columns x R rows (R = 2^LOG_R), TC R / 16 threads, thread
// (c = tid % TC, r0 = tid / TC).  in: v[k] = row r0 + (R / 16) k; out: v[k] = row 16 r0 + k; lds: R TC doubles (unused for
// R = 16, where one register pass does everything and rows k go in and out).  Growth: at most 0.51 p per stage.
template <int LOG_R, int TC = (4096 >> LOG_R)>
__device__ __forceinline__ void col_fwd_core(double (&v)[16], const PassTwiddles& t, uint32_t c, uint32_t r0, double* lds, Mod m) {
    constexpr int E = LOG_R - 4, S = 1 << E;
    radix16_fwd(v, t.a, m);
    if constexpr (E > 0) {
#pragma unroll
        for (int k = 0; k < 16; ++k) lds[(r0 + S * k) * TC + c] = v[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = lds[(16 * r0 + k) * TC + c];
        radix16_fwd<4 - E>(v, t.b, m);
    }
}

// Last log2(R) inverse stages on a column tile (no N^-1 factor): in rows 16 r0 + k, out rows r0 + (R / 16) k.
// in: |v| <= p.  out: |v| <= 16 p.
template <int LOG_R, int TC = (4096 >> LOG_R)>
__device__ __forceinline__ void col_inv_core(double (&v)[16], const PassTwiddles& t, uint32_t c, uint32_t r0, double* lds, Mod m) {
    constexpr int E = LOG_R - 4, S = 1 << E;
    if constexpr (E > 0) {
        radix16_inv<4 - E>(v, t.b, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) lds[(16 * r0 + k) * TC + c] = reduce_lazy(v[k], m);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = lds[(r0 + S * k) * TC + c];
    }
    radix16_inv(v, t.a, m);
}

// Buffer descriptor of a tensor slice (raw, unstrided; gfx9 data-format word): loads through it take a per-lane byte
// offset in a vector register plus a uniform byte offset in a scalar register, and reads beyond `bytes` return zero.
using BufferRsrc = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ BufferRsrc make_buffer_rsrc(const void* base, uint64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(uint32_t)bytes, 0x00020000);
}

// Point k of the 16 strided points of a column-pass thread (rows r0 + (R / 16) k): the double at byte offset
// limb_off + k * 16 R * 8 + lane_off of the buffer, lane_off = 8 (256 r0 + column).
template <int LOG_R>
__device__ __forceinline__ double load_strided_point(BufferRsrc rsrc, uint32_t lane_off, uint32_t limb_off, int k) {
    constexpr uint32_t kStrideBytes = (16u << LOG_R) * 8u;
    return __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_off, (int)(limb_off + k * kStrideBytes), 0));
}

// Row index of v[k] before / after the column cores, and the first column of the tile.
template <int LOG_R>
__device__ __forceinline__ uint32_t col_row_strided(uint32_t r0, int k) { return r0 + ((uint32_t)k << (LOG_R - 4)); }
template <int LOG_R>
__device__ __forceinline__ uint32_t col_row_grouped(uint32_t r0, int k) { return 16 * r0 + (uint32_t)k; }

}  // namespace ks
