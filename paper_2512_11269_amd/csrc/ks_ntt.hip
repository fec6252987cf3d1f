// Negacyclic NTT / INTT for N = 2^12 .. 2^16 (Background, "NTT"; Kernel Code Generation, NTT kernels).
//
// A limb is viewed as an R x 256 matrix (row-major, R = N / 256).  The forward transform runs its first
// log2(R) decimation-in-time stages down the columns (butterfly partners R/2 ... 1 rows apart) and its last
// 8 stages inside the contiguous 256-point rows; the inverse mirrors it.  Each thread owns 16 points: four
// stages run in registers, then the tile is re-distributed through LDS for the next (up to) four.  Intermediate
// results between the two kernels of a transform are raw doubles (lazy representatives); only the last
// kernel reduces to canonical residues.
#include <algorithm>

#include "ks_internal.hpp"
#include "ks_tasks.hpp"

namespace ks {

struct LimbRef {
    const uint64_t* in;
    uint64_t* out;
    uint32_t mod_id, idx;
};

__device__ __forceinline__ LimbRef locate(const LimbMap& map, uint32_t li, const uint64_t* in, uint64_t* out,
                                          uint64_t in_ps, uint64_t out_ps, uint32_t N) {
    const uint32_t poly = li / map.n, idx = li - poly * map.n;
    const uint64_t off = (uint64_t)map.off[idx] * N;
    return LimbRef{in + poly * in_ps + off, out + poly * out_ps + off, map.mod[idx], idx};
}

// forward, columns: canonical u64 in, raw doubles out (|x| <= (1 + 0.501 log2 R) p).
template <int LOG_R, int TC>
__global__ __launch_bounds__((TC << LOG_R) / 16) void ntt_fwd_cols(const double* __restrict__ tw, const Mod* __restrict__ mods, LimbMap map,
                                                        const uint64_t* in, uint64_t* out, uint64_t in_ps, uint64_t out_ps) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 256 / TC;
    __shared__ double lds[LOG_R > 4 ? (TC << LOG_R) : 1];
    const uint32_t tid = threadIdx.x;
    const uint32_t li = blockIdx.x / TILES, tile = blockIdx.x - li * TILES;
    const LimbRef L = locate(map, li, in, out, in_ps, out_ps, N);
    const Mod m = mods[L.mod_id];
    const double* W = tw + (size_t)L.mod_id * N;
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = u64_to_f64(L.in[col_row_strided<LOG_R>(r0, k) * 256 + col]);
    load_col_twiddles<LOG_R>(t, W, r0);
    col_fwd_core<LOG_R, TC>(v, t, c, r0, lds, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) store_f64(L.out + col_row_grouped<LOG_R>(r0, k) * 256 + col, v[k]);
}

// forward, rows, in place: raw doubles in, canonical residues out.  One wavefront = four rows.
template <int LOG_R>
__global__ __launch_bounds__(64) void ntt_fwd_rows(TwTables tw, const Mod* __restrict__ mods, LimbMap map, uint64_t* data, uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, GROUPS = R / 4;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t tid = threadIdx.x;
    const uint32_t li = blockIdx.x / GROUPS, rg = blockIdx.x - li * GROUPS;
    const uint32_t poly = li / map.n, idx = li - poly * map.n, mod_id = map.mod[idx];
    const Mod m = mods[mod_id];
    const uint32_t j0 = tid & 15, rr = tid >> 4, row = rg * 4 + rr;
    uint64_t* p = data + poly * ps + (uint64_t)map.off[idx] * N + row * 256;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load_f64(p + j0 + 16 * k);
    load_row_twiddles(t, tw, mod_id, N, R + row, j0, m);
    row_fwd_core(v, t, j0, lds + rr * kRowPitch, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) p[j0 + 16 * k] = f64_to_u64(canon(reduce_lazy(v[k], m), m));
}

// The bundle [b][ndig][E][N] the rotation gathers read, finished in one launch.  The first n_new_blocks workgroups run the
// row half of the forward transform on the raised limbs (`lifted`, the same element layout, raw doubles after the column
// half) and write canonical residues; the others copy the polynomial's own limbs d[b][pos] (WD words, d_ps apart) into
// the slots (b, digit of pos, pos), so that every slot of the bundle is filled and a gather needs no own / raised
// distinction.  PACKED: bits 0..31 of a residue go to the 32-bit word array lo and the bits above (moduli are below 2^36)
// to the byte array hi with the same element index, 5 bytes a residue instead of 8; a transforming thread then ends with
// sixteen consecutive points and stores them as four 16-byte words plus one 16-byte word of high bytes, so the row needs
// no last exchange through LDS.  Otherwise (moduli below 2^32) lo alone holds 32-bit words.
template <int LOG_R, bool PACKED, typename WD>
__global__ __launch_bounds__(64) void gather_bundle_rows(TwTables tw, const Mod* __restrict__ mods, LimbMap map, DigitRanges dg,
                                                         uint32_t ell, uint32_t E, const uint64_t* __restrict__ lifted,
                                                         const WD* __restrict__ d, uint64_t d_ps, uint32_t n_new_blocks,
                                                         uint32_t* __restrict__ lo, uint8_t* __restrict__ hi) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, GROUPS = R / 4;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t tid = threadIdx.x, j0 = tid & 15, rr = tid >> 4;
    const uint64_t ps = (uint64_t)dg.ndig * E * N;
    if (blockIdx.x >= n_new_blocks) {  // uniform: copy four rows of an own limb
        const uint32_t t = blockIdx.x - n_new_blocks, li = t / GROUPS, row = (t - li * GROUPS) * 4 + rr;
        const uint32_t poly = li / ell, pos = li - poly * ell;
        uint32_t j = 0;
        while (j + 1 < dg.ndig && pos >= dg.hi[j]) ++j;  // uniform
        const WD* src = d + poly * d_ps + (uint64_t)pos * N + row * 256 + j0;
        const uint64_t e = poly * ps + ((uint64_t)j * E + pos) * N + row * 256 + j0;
        WD u[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) u[k] = src[16 * k];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            lo[e + 16 * k] = (uint32_t)u[k];
            if constexpr (PACKED) hi[e + 16 * k] = (uint8_t)((uint64_t)u[k] >> 32);
        }
        return;
    }
    const uint32_t li = blockIdx.x / GROUPS, rg = blockIdx.x - li * GROUPS;
    const uint32_t poly = li / map.n, idx = li - poly * map.n, mod_id = map.mod[idx];
    const uint64_t off = poly * ps + (uint64_t)map.off[idx] * N;
    const Mod m = mods[mod_id];
    const uint32_t row = rg * 4 + rr;
    const uint64_t* ip = lifted + off + row * 256;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load_f64(ip + j0 + 16 * k);
    load_row_twiddles(t, tw, mod_id, N, R + row, j0, m);
    if constexpr (PACKED) {
        row_fwd_core_consecutive(v, t, j0, lds + rr * kRowPitch, m);
        uint32_t l[16], h[4] = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint64_t u = f64_to_u64(canon(reduce_lazy(v[k], m), m));
            l[k] = (uint32_t)u;
            h[k >> 2] |= (uint32_t)(u >> 32) << (8 * (k & 3));
        }
        const uint64_t e = off + row * 256 + 16 * j0;
        uint4* lp = reinterpret_cast<uint4*>(lo + e);
#pragma unroll
        for (int q = 0; q < 4; ++q) lp[q] = make_uint4(l[4 * q], l[4 * q + 1], l[4 * q + 2], l[4 * q + 3]);
        *reinterpret_cast<uint4*>(hi + e) = make_uint4(h[0], h[1], h[2], h[3]);
    } else {
        row_fwd_core(v, t, j0, lds + rr * kRowPitch, m);
        uint32_t* op = lo + off + row * 256 + j0;
#pragma unroll
        for (int k = 0; k < 16; ++k) op[16 * k] = (uint32_t)canon(reduce_lazy(v[k], m), m);
    }
}

// inverse, rows first: canonical residues in (64- or 32-bit words), raw doubles out (|x| <= 0.501 p).
template <int LOG_R, typename W>
__global__ __launch_bounds__(64) void ntt_inv_rows(TwTables twi, const Mod* __restrict__ mods, LimbMap map,
                                                   const W* in, uint64_t* out, uint64_t in_ps, uint64_t out_ps) {
    constexpr uint32_t N = 256u << LOG_R, GROUPS = (1u << LOG_R) / 4;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t li = blockIdx.x / GROUPS, rg = blockIdx.x - li * GROUPS;
    const uint32_t poly = li / map.n, idx = li - poly * map.n, mod_id = map.mod[idx];
    const uint64_t off = (uint64_t)map.off[idx] * N;
    task_inv_rows<LOG_R, W>(twi, mods[mod_id], mod_id, in + poly * in_ps + off, out + poly * out_ps + off, rg, threadIdx.x, lds);
}

// inverse, columns last, in place: raw doubles in; out = canonical [x * scale]_m where scale is N^-1,
// optionally pre-multiplied by a per-limb constant (base conversion folds its (D/s_i)^-1 in here).
// OUT_F64: store the canonical result as a double instead of a 64-bit integer.
template <int LOG_R, int TC, bool OUT_F64>
__global__ __launch_bounds__((TC << LOG_R) / 16) void ntt_inv_cols(const double* __restrict__ twi, const Mod* __restrict__ mods,
                                                        const double* __restrict__ scale_tab, int scale_by_idx, LimbMap map,
                                                        uint64_t* data, uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 256 / TC;
    __shared__ double lds[LOG_R > 4 ? (TC << LOG_R) : 1];
    const uint32_t li = blockIdx.x / TILES, tile = blockIdx.x - li * TILES;
    const LimbRef L = locate(map, li, data, data, ps, ps, N);
    task_inv_cols<LOG_R, TC, OUT_F64>(twi + (size_t)L.mod_id * N, mods[L.mod_id], scale_tab[scale_by_idx ? L.idx : L.mod_id], L.in,
                                      L.out, tile, threadIdx.x, lds);
}

// ------------------------------------------------------------------------------------------------
// Transforms of limbs held in 32-bit words (every modulus below 2^32), in place.  Both passes read and write canonical
// residues, so the half-way values fit the same words and a transform moves half the bytes of the 64-bit one.
// fwd_cols -> fwd_rows, inv_rows -> inv_cols as above.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t* locate_u32(const LimbMap& map, uint32_t li, uint32_t* data, uint64_t ps, uint32_t N,
                                                uint32_t* mod_id) {
    const uint32_t poly = li / map.n, idx = li - poly * map.n;
    *mod_id = map.mod[idx];
    return data + poly * ps + (uint64_t)map.off[idx] * N;
}

template <int LOG_R, int TC>
__global__ __launch_bounds__((TC << LOG_R) / 16) void ntt_fwd_cols_u32(const double* __restrict__ tw, const Mod* __restrict__ mods,
                                                                     LimbMap map, uint32_t* data, uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 256 / TC;
    __shared__ double lds[LOG_R > 4 ? (TC << LOG_R) : 1];
    const uint32_t tid = threadIdx.x, li = blockIdx.x / TILES, tile = blockIdx.x - li * TILES;
    uint32_t mod_id;
    uint32_t* p = locate_u32(map, li, data, ps, N, &mod_id);
    const Mod m = mods[mod_id];
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = (double)p[col_row_strided<LOG_R>(r0, k) * 256 + col];
    load_col_twiddles<LOG_R>(t, tw + (size_t)mod_id * N, r0);
    col_fwd_core<LOG_R, TC>(v, t, c, r0, lds, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) p[col_row_grouped<LOG_R>(r0, k) * 256 + col] = (uint32_t)canon(reduce_lazy(v[k], m), m);
}

template <int LOG_R, bool INVERSE>
__global__ __launch_bounds__(64) void ntt_rows_u32(TwTables tw, const Mod* __restrict__ mods, LimbMap map, uint32_t* data,
                                                   uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, GROUPS = R / 4;
    __shared__ double lds[4 * kRowPitch];
    const uint32_t tid = threadIdx.x, li = blockIdx.x / GROUPS, rg = blockIdx.x - li * GROUPS;
    uint32_t mod_id;
    uint32_t* limb = locate_u32(map, li, data, ps, N, &mod_id);
    const Mod m = mods[mod_id];
    const uint32_t j0 = tid & 15, rr = tid >> 4, row = rg * 4 + rr;
    uint32_t* p = limb + row * 256;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = (double)p[j0 + 16 * k];
    load_row_twiddles(t, tw, mod_id, N, R + row, j0, m);
    if constexpr (INVERSE) row_inv_core(v, t, j0, lds + rr * kRowPitch, m);
    else row_fwd_core(v, t, j0, lds + rr * kRowPitch, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) p[j0 + 16 * k] = (uint32_t)canon(reduce_lazy(v[k], m), m);
}

template <int LOG_R, int TC>
__global__ __launch_bounds__((TC << LOG_R) / 16) void ntt_inv_cols_u32(const double* __restrict__ twi, const Mod* __restrict__ mods,
                                                                     const double* __restrict__ ninv, LimbMap map, uint32_t* data,
                                                                     uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, TILES = 256 / TC;
    __shared__ double lds[LOG_R > 4 ? (TC << LOG_R) : 1];
    const uint32_t tid = threadIdx.x, li = blockIdx.x / TILES, tile = blockIdx.x - li * TILES;
    uint32_t mod_id;
    uint32_t* p = locate_u32(map, li, data, ps, N, &mod_id);
    const Mod m = mods[mod_id];
    const double scale = ninv[mod_id];
    const uint32_t c = tid & (TC - 1), r0 = tid / TC, col = tile * TC + c;
    double v[16];
    PassTwiddles t;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = (double)p[col_row_grouped<LOG_R>(r0, k) * 256 + col];
    load_col_twiddles<LOG_R>(t, twi + (size_t)mod_id * N, r0);
    col_inv_core<LOG_R, TC>(v, t, c, r0, lds, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) p[col_row_strided<LOG_R>(r0, k) * 256 + col] = (uint32_t)canon(mulmod_lazy(v[k], scale, m), m);
}

// ------------------------------------------------------------------------------------------------
// Wide tiles (32 columns, 256-byte segments) move more bytes per second but give half as many workgroups;
// small launches keep the 16-column tiles.
static bool wide_tiles(uint32_t limbs) { return limbs >= 256; }

void launch_ntt_fwd_cols(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s) {
    const uint32_t limbs = map.n * io.n_polys;
    if (limbs == 0) return;
    const uint64_t* in = static_cast<const uint64_t*>(io.in);
    uint64_t* out = static_cast<uint64_t*>(io.out);
    ProfScope ps("ntt_fwd_cols", 2.0 * limbs * c->N * 8.0, s);
    if (c->logN == 16 && wide_tiles(limbs)) {
        hipLaunchKernelGGL((ntt_fwd_cols<8, 32>), dim3(limbs * 8), dim3(512), 0, s, c->d_tw_fwd, c->d_mod, map, in, out,
                           io.in_poly_stride, io.out_poly_stride);
        return;
    }
#define KS_LAUNCH(LOGR)                                                                                                          \
    hipLaunchKernelGGL((ntt_fwd_cols<LOGR, (4096 >> LOGR)>), dim3(limbs << (LOGR - 4)), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, map, in, \
                       out, io.in_poly_stride, io.out_poly_stride)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
}

void launch_ntt_fwd_rows(const ks_ctx* c, const LimbMap& map, uint64_t* data, uint64_t ps_words, uint32_t n_polys, hipStream_t s) {
    const uint32_t limbs = map.n * n_polys;
    if (limbs == 0) return;
    ProfScope ps("ntt_fwd_rows", 2.0 * limbs * c->N * 8.0, s);
#define KS_LAUNCH(LOGR) \
    hipLaunchKernelGGL((ntt_fwd_rows<LOGR>), dim3(limbs << (LOGR - 2)), dim3(64), 0, s, c->tw_fwd, c->d_mod, map, data, ps_words)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
}

void launch_gather_bundle_rows(const ks_ctx* c, const Level& lv, const uint64_t* lifted, const void* d, uint64_t d_ps, bool d_words32,
                               const PackedDigits& out, uint32_t n_polys, hipStream_t s) {
    if (n_polys == 0) return;
    const uint32_t n_new = lv.lifted_map.n * n_polys, n_own = lv.ell * n_polys;
    DigitRanges dg;
    dg.ndig = lv.ndig;
    for (uint32_t j = 0; j < kMaxDigits; ++j) {
        dg.lo[j] = j < lv.ndig ? lv.digit_lo[j] : 0;
        dg.hi[j] = j < lv.ndig ? lv.digit_hi[j] : 0;
    }
    const double wb = out.hi ? 5.0 : 4.0;
    ProfScope ps("gather_bundle_rows", ((8.0 + wb) * n_new + ((d_words32 ? 4.0 : 8.0) + wb) * n_own) * c->N, s);
#define KS_LAUNCH(LOGR)                                                                                                              \
    if (out.hi)                                                                                                                      \
        hipLaunchKernelGGL((gather_bundle_rows<LOGR, true, uint64_t>), dim3((n_new + n_own) << (LOGR - 2)), dim3(64), 0, s, c->tw_fwd, \
                           c->d_mod, lv.lifted_map, dg, lv.ell, lv.E, lifted, static_cast<const uint64_t*>(d), d_ps,                 \
                           n_new << (LOGR - 2), out.lo, out.hi);                                                                     \
    else                                                                                                                             \
        hipLaunchKernelGGL((gather_bundle_rows<LOGR, false, uint32_t>), dim3((n_new + n_own) << (LOGR - 2)), dim3(64), 0, s, c->tw_fwd, \
                           c->d_mod, lv.lifted_map, dg, lv.ell, lv.E, lifted, static_cast<const uint32_t*>(d), d_ps,                 \
                           n_new << (LOGR - 2), out.lo, out.hi)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
}

// Polynomials per launch pair of a two-pass transform: the second pass of a group should find what the first pass wrote
// still in the 256 MB last-level cache.  Measured on 1920 limbs: groups of 240 MB are 8 % faster than one pair of launches
// over everything, groups of 64 MB 9 % slower (launches too small), groups of 320 MB no different.
static uint32_t polys_per_group(const ks_ctx* c, const LimbMap& map) {
    constexpr uint64_t kGroupBytes = 240ull << 20;
    const uint64_t poly_bytes = (uint64_t)map.n * c->N * 8;
    return (uint32_t)std::max<uint64_t>(1, kGroupBytes / poly_bytes);
}

void launch_ntt_fwd(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s) {
    const uint32_t g = polys_per_group(c, map);
    for (uint32_t p0 = 0; p0 < io.n_polys; p0 += g) {
        const uint32_t np = std::min(g, io.n_polys - p0);
        XformIO part{static_cast<const uint64_t*>(io.in) + (uint64_t)p0 * io.in_poly_stride,
                     static_cast<uint64_t*>(io.out) + (uint64_t)p0 * io.out_poly_stride, io.in_poly_stride, io.out_poly_stride, np};
        launch_ntt_fwd_cols(c, map, part, s);
        launch_ntt_fwd_rows(c, map, static_cast<uint64_t*>(part.out), io.out_poly_stride, np, s);
    }
}

void launch_ntt_inv_rows(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s, bool in_words32) {
    const uint32_t limbs = map.n * io.n_polys;
    if (limbs == 0) return;
    uint64_t* out = static_cast<uint64_t*>(io.out);
    ProfScope ps("ntt_inv_rows", (in_words32 ? 1.5 : 2.0) * limbs * c->N * 8.0, s);
#define KS_LAUNCH(LOGR)                                                                                                          \
    if (in_words32)                                                                                                              \
        hipLaunchKernelGGL((ntt_inv_rows<LOGR, uint32_t>), dim3(limbs << (LOGR - 2)), dim3(64), 0, s, c->tw_inv, c->d_mod, map,          \
                           static_cast<const uint32_t*>(io.in), out, io.in_poly_stride, io.out_poly_stride);                     \
    else                                                                                                                         \
        hipLaunchKernelGGL((ntt_inv_rows<LOGR, uint64_t>), dim3(limbs << (LOGR - 2)), dim3(64), 0, s, c->tw_inv, c->d_mod, map,          \
                           static_cast<const uint64_t*>(io.in), out, io.in_poly_stride, io.out_poly_stride)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
}

void launch_ntt_inv_cols(const ks_ctx* c, const LimbMap& map, uint64_t* data, uint64_t ps_words, uint32_t n_polys,
                         const double* scale_tab, bool scale_by_idx, bool out_f64, hipStream_t s) {
    const uint32_t limbs = map.n * n_polys;
    if (limbs == 0) return;
    ProfScope ps("ntt_inv_cols", 2.0 * limbs * c->N * 8.0, s);
    const int by_idx = scale_by_idx ? 1 : 0;
#define KS_LAUNCH_INV_COLS(LOGR, TCV, GRID, F64)                                                                               \
    hipLaunchKernelGGL((ntt_inv_cols<LOGR, TCV, F64>), dim3(GRID), dim3((TCV << LOGR) / 16), 0, s, c->d_tw_inv, c->d_mod, scale_tab, \
                       by_idx, map, data, ps_words)
    if (c->logN == 16 && wide_tiles(limbs)) {
        if (out_f64) KS_LAUNCH_INV_COLS(8, 32, limbs * 8, true);
        else KS_LAUNCH_INV_COLS(8, 32, limbs * 8, false);
        return;
    }
#define KS_LAUNCH(LOGR)                                                                       \
    if (out_f64) KS_LAUNCH_INV_COLS(LOGR, (4096 >> LOGR), limbs << (LOGR - 4), true); \
    else KS_LAUNCH_INV_COLS(LOGR, (4096 >> LOGR), limbs << (LOGR - 4), false)
    KS_FOR_LOG_R(c->logN, KS_LAUNCH)
#undef KS_LAUNCH
#undef KS_LAUNCH_INV_COLS
}

void launch_ntt_inv(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s) {
    const uint32_t g = polys_per_group(c, map);
    for (uint32_t p0 = 0; p0 < io.n_polys; p0 += g) {
        const uint32_t np = std::min(g, io.n_polys - p0);
        XformIO part{static_cast<const uint64_t*>(io.in) + (uint64_t)p0 * io.in_poly_stride,
                     static_cast<uint64_t*>(io.out) + (uint64_t)p0 * io.out_poly_stride, io.in_poly_stride, io.out_poly_stride, np};
        launch_ntt_inv_rows(c, map, part, s);
        launch_ntt_inv_cols(c, map, static_cast<uint64_t*>(part.out), io.out_poly_stride, np, c->d_ninv, false, false, s);
    }
}

void launch_ntt_u32(const ks_ctx* c, const LimbMap& map, uint32_t* data, uint64_t ps_words, uint32_t n_polys, bool inverse,
                    hipStream_t s) {
    // groups sized like the 64-bit transform's: the second pass should find the first pass's output in the last-level cache
    const uint32_t g = 2 * polys_per_group(c, map);
    for (uint32_t p0 = 0; p0 < n_polys; p0 += g) {
        const uint32_t limbs = map.n * std::min(g, n_polys - p0);
        uint32_t* part = data + (uint64_t)p0 * ps_words;
        // column tiles: 32 columns at N = 2^16 (128-byte row segments of 32-bit words), 4096 / R otherwise
#define KS_LAUNCH_TC(LOGR, TCV)                                                                                                     \
    if (!inverse) {                                                                                                                 \
        {                                                                                                                           \
            ProfScope ps("ntt_fwd_cols_u32", 1.0 * limbs * c->N * 8.0, s);                                                          \
            hipLaunchKernelGGL((ntt_fwd_cols_u32<LOGR, TCV>), dim3(limbs * (256 / TCV)), dim3((TCV << LOGR) / 16), 0, s,            \
                               c->d_tw_fwd, c->d_mod, map, part, ps_words);                                                        \
        }                                                                                                                           \
        ProfScope ps("ntt_fwd_rows_u32", 1.0 * limbs * c->N * 8.0, s);                                                              \
        hipLaunchKernelGGL((ntt_rows_u32<LOGR, false>), dim3(limbs << (LOGR - 2)), dim3(64), 0, s, c->tw_fwd, c->d_mod, map, part,  \
                           ps_words);                                                                                              \
    } else {                                                                                                                        \
        {                                                                                                                           \
            ProfScope ps("ntt_inv_rows_u32", 1.0 * limbs * c->N * 8.0, s);                                                          \
            hipLaunchKernelGGL((ntt_rows_u32<LOGR, true>), dim3(limbs << (LOGR - 2)), dim3(64), 0, s, c->tw_inv, c->d_mod, map,     \
                               part, ps_words);                                                                                    \
        }                                                                                                                           \
        ProfScope ps("ntt_inv_cols_u32", 1.0 * limbs * c->N * 8.0, s);                                                              \
        hipLaunchKernelGGL((ntt_inv_cols_u32<LOGR, TCV>), dim3(limbs * (256 / TCV)), dim3((TCV << LOGR) / 16), 0, s, c->d_tw_inv,   \
                           c->d_mod, c->d_ninv, map, part, ps_words);                                                              \
    }
        switch (c->logN) {
            case 12: KS_LAUNCH_TC(4, 256) break;
            case 13: KS_LAUNCH_TC(5, 128) break;
            case 14: KS_LAUNCH_TC(6, 64) break;
            case 15: KS_LAUNCH_TC(7, 32) break;
            default: KS_LAUNCH_TC(8, 32) break;
        }
#undef KS_LAUNCH_TC
    }
}

}  // namespace ks
