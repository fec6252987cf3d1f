// Negacyclic NTT / INTT for N = 2^12 and 2^16 (Background, "NTT"; Kernel Code Generation, NTT kernels).
//
// A limb is viewed as an R x 256 matrix (row-major, R = N / 256).  The forward transform runs its first
// log2(R) decimation-in-time stages down the columns ("phase A", butterfly partners R/2 ... 1 rows apart)
// and its last 8 stages inside the contiguous 256-point rows ("phase B").  Each workgroup of 256 threads
// owns a 4096-point tile, each thread 16 points: four stages run in registers, then the tile is
// re-distributed through LDS for the next four.  Intermediate results between the phases are stored as raw
// doubles (lazy representatives); only the last phase reduces to canonical residues.
//
// Twiddles: one table per modulus, W[k] = psi^brv(k) (heap order: the stage with 2^s blocks uses
// W[2^s .. 2^(s+1)-1]), so the 15 twiddles of a 16-point register pass are the sub-tree below one node.
#include "ks_internal.hpp"

namespace ks {

constexpr int kRowPitch = 272;  // 256 points + 1 pad per 16: transposed LDS reads hit distinct banks

__device__ __forceinline__ double load_elem_u64(const uint64_t* p) { return u64_to_f64(*p); }
__device__ __forceinline__ double load_elem_f64(const uint64_t* p) { return *reinterpret_cast<const double*>(p); }
__device__ __forceinline__ void store_elem_f64(uint64_t* p, double v) { *reinterpret_cast<double*>(p) = v; }

struct LimbRef {
    const uint64_t* in;
    uint64_t* out;
    uint32_t mod_id;
};

__device__ __forceinline__ LimbRef locate(const LimbMap& map, uint32_t li, const uint64_t* in, uint64_t* out,
                                          uint64_t in_ps, uint64_t out_ps, uint32_t N) {
    const uint32_t poly = li / map.n, idx = li - poly * map.n;
    const uint64_t off = (uint64_t)map.off[idx] * N;
    return LimbRef{in + poly * in_ps + off, out + poly * out_ps + off, map.mod[idx]};
}

// ------------------------------------------------------------------------------------------------
// forward, phase A: columns.  LOG_R = 8: tile = 16 columns x 256 rows; LOG_R = 4: tile = 256 x 16 rows.
// in: canonical u64.  out: raw doubles, magnitude <= (1 + 0.501 LOG_R) p.
// ------------------------------------------------------------------------------------------------
template <int LOG_R>
__global__ __launch_bounds__(256) void ntt_fwd_cols(const double* __restrict__ tw, const Mod* __restrict__ mods, LimbMap map,
                                                    const uint64_t* in, uint64_t* out, uint64_t in_ps, uint64_t out_ps) {
    constexpr uint32_t N = 256u << LOG_R;
    const uint32_t tid = threadIdx.x;
    double v[16];
    if constexpr (LOG_R == 8) {
        __shared__ double lds[4096];
        const uint32_t tile = blockIdx.x & 15, li = blockIdx.x >> 4;
        const LimbRef L = locate(map, li, in, out, in_ps, out_ps, N);
        const Mod m = mods[L.mod_id];
        const double* W = tw + (size_t)L.mod_id * N;
        const uint32_t c = tid & 15, r0 = tid >> 4, col = tile * 16 + c;
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = load_elem_u64(L.in + (r0 + 16 * k) * 256 + col);
        radix16_fwd(v, W, 1, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) lds[(r0 + 16 * k) * 16 + c] = v[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = lds[(16 * r0 + k) * 16 + c];
        radix16_fwd(v, W, 16 + r0, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) store_elem_f64(L.out + (16 * r0 + k) * 256 + col, v[k]);
    } else {
        const LimbRef L = locate(map, blockIdx.x, in, out, in_ps, out_ps, N);
        const Mod m = mods[L.mod_id];
        const double* W = tw + (size_t)L.mod_id * N;
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = load_elem_u64(L.in + k * 256 + tid);
        radix16_fwd(v, W, 1, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) store_elem_f64(L.out + k * 256 + tid, v[k]);
    }
}

// ------------------------------------------------------------------------------------------------
// forward, phase B: 16 contiguous rows of 256 points per workgroup.  in: raw doubles (|x| <= 7 p),
// out: canonical u64.
// ------------------------------------------------------------------------------------------------
template <int LOG_R>
__global__ __launch_bounds__(256) void ntt_fwd_rows(const double* __restrict__ tw, const Mod* __restrict__ mods, LimbMap map,
                                                    uint64_t* data, uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, TILES = R / 16;
    __shared__ double lds[16 * kRowPitch];
    const uint32_t tid = threadIdx.x;
    const uint32_t li = blockIdx.x / TILES, rt = blockIdx.x - li * TILES;
    const LimbRef L = locate(map, li, data, data, ps, ps, N);
    const Mod m = mods[L.mod_id];
    const double* W = tw + (size_t)L.mod_id * N;
    const uint32_t j0 = tid & 15, rr = tid >> 4, row = rt * 16 + rr;
    uint64_t* p = L.out + row * 256;
    double* lrow = lds + rr * kRowPitch;
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load_elem_f64(p + j0 + 16 * k);
    radix16_fwd(v, W, R + row, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_fwd(v, W, (R + row) * 16 + j0, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[17 * j0 + k] = canon(reduce_lazy(v[k], m), m);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) p[j0 + 16 * k] = f64_to_u64(lrow[j0 + 17 * k]);
}

// ------------------------------------------------------------------------------------------------
// inverse, phase B first: rows.  in: canonical u64, out: raw doubles with |x| <= 0.501 p.
// ------------------------------------------------------------------------------------------------
template <int LOG_R>
__global__ __launch_bounds__(256) void ntt_inv_rows(const double* __restrict__ twi, const Mod* __restrict__ mods, LimbMap map,
                                                    const uint64_t* in, uint64_t* out, uint64_t in_ps, uint64_t out_ps) {
    constexpr uint32_t N = 256u << LOG_R, R = 1u << LOG_R, TILES = R / 16;
    __shared__ double lds[16 * kRowPitch];
    const uint32_t tid = threadIdx.x;
    const uint32_t li = blockIdx.x / TILES, rt = blockIdx.x - li * TILES;
    const LimbRef L = locate(map, li, in, out, in_ps, out_ps, N);
    const Mod m = mods[L.mod_id];
    const double* Wi = twi + (size_t)L.mod_id * N;
    const uint32_t j0 = tid & 15, rr = tid >> 4, row = rt * 16 + rr;
    double* lrow = lds + rr * kRowPitch;
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[j0 + 17 * k] = load_elem_u64(L.in + row * 256 + j0 + 16 * k);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[17 * j0 + k];
    radix16_inv(v, Wi, (R + row) * 16 + j0, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) lrow[17 * j0 + k] = reduce_lazy(v[k], m);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = lrow[j0 + 17 * k];
    radix16_inv(v, Wi, R + row, m);
#pragma unroll
    for (int k = 0; k < 16; ++k) store_elem_f64(L.out + row * 256 + j0 + 16 * k, reduce_lazy(v[k], m));
}

// ------------------------------------------------------------------------------------------------
// inverse, phase A last: columns, then multiply by N^-1.  in place: raw doubles -> canonical u64.
// ------------------------------------------------------------------------------------------------
template <int LOG_R>
__global__ __launch_bounds__(256) void ntt_inv_cols(const double* __restrict__ twi, const Mod* __restrict__ mods,
                                                    const double* __restrict__ ninv, LimbMap map, uint64_t* data, uint64_t ps) {
    constexpr uint32_t N = 256u << LOG_R;
    const uint32_t tid = threadIdx.x;
    double v[16];
    if constexpr (LOG_R == 8) {
        __shared__ double lds[4096];
        const uint32_t tile = blockIdx.x & 15, li = blockIdx.x >> 4;
        const LimbRef L = locate(map, li, data, data, ps, ps, N);
        const Mod m = mods[L.mod_id];
        const double* Wi = twi + (size_t)L.mod_id * N;
        const double scale = ninv[L.mod_id];
        const uint32_t c = tid & 15, r0 = tid >> 4, col = tile * 16 + c;
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = load_elem_f64(L.in + (16 * r0 + k) * 256 + col);
        radix16_inv(v, Wi, 16 + r0, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) lds[(16 * r0 + k) * 16 + c] = reduce_lazy(v[k], m);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = lds[(r0 + 16 * k) * 16 + c];
        radix16_inv(v, Wi, 1, m);
#pragma unroll
        for (int k = 0; k < 16; ++k)
            L.out[(r0 + 16 * k) * 256 + col] = f64_to_u64(canon(mulmod_lazy(v[k], scale, m), m));
    } else {
        const LimbRef L = locate(map, blockIdx.x, data, data, ps, ps, N);
        const Mod m = mods[L.mod_id];
        const double* Wi = twi + (size_t)L.mod_id * N;
        const double scale = ninv[L.mod_id];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = load_elem_f64(L.in + k * 256 + tid);
        radix16_inv(v, Wi, 1, m);
#pragma unroll
        for (int k = 0; k < 16; ++k) L.out[k * 256 + tid] = f64_to_u64(canon(mulmod_lazy(v[k], scale, m), m));
    }
}

// ------------------------------------------------------------------------------------------------
void launch_ntt_fwd(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s) {
    const uint32_t limbs = map.n * io.n_polys;
    if (limbs == 0) return;
    const uint64_t* in = static_cast<const uint64_t*>(io.in);
    uint64_t* out = static_cast<uint64_t*>(io.out);
    const double bytes = 2.0 * limbs * c->N * 8.0;
    if (c->logN == 16) {
        { ProfScope ps("ntt_fwd_cols", bytes, s);
        hipLaunchKernelGGL(ntt_fwd_cols<8>, dim3(limbs * 16), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, map, in, out,
                           io.in_poly_stride, io.out_poly_stride); }
        { ProfScope ps("ntt_fwd_rows", bytes, s);
        hipLaunchKernelGGL(ntt_fwd_rows<8>, dim3(limbs * 16), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, map, out,
                           io.out_poly_stride); }
    } else {
        { ProfScope ps("ntt_fwd_cols", bytes, s);
        hipLaunchKernelGGL(ntt_fwd_cols<4>, dim3(limbs), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, map, in, out,
                           io.in_poly_stride, io.out_poly_stride); }
        { ProfScope ps("ntt_fwd_rows", bytes, s);
        hipLaunchKernelGGL(ntt_fwd_rows<4>, dim3(limbs), dim3(256), 0, s, c->d_tw_fwd, c->d_mod, map, out,
                           io.out_poly_stride); }
    }
}

void launch_ntt_inv(const ks_ctx* c, const LimbMap& map, const XformIO& io, hipStream_t s) {
    const uint32_t limbs = map.n * io.n_polys;
    if (limbs == 0) return;
    const uint64_t* in = static_cast<const uint64_t*>(io.in);
    uint64_t* out = static_cast<uint64_t*>(io.out);
    const double bytes = 2.0 * limbs * c->N * 8.0;
    if (c->logN == 16) {
        { ProfScope ps("ntt_inv_rows", bytes, s);
        hipLaunchKernelGGL(ntt_inv_rows<8>, dim3(limbs * 16), dim3(256), 0, s, c->d_tw_inv, c->d_mod, map, in, out,
                           io.in_poly_stride, io.out_poly_stride); }
        { ProfScope ps("ntt_inv_cols", bytes, s);
        hipLaunchKernelGGL(ntt_inv_cols<8>, dim3(limbs * 16), dim3(256), 0, s, c->d_tw_inv, c->d_mod, c->d_ninv, map, out,
                           io.out_poly_stride); }
    } else {
        { ProfScope ps("ntt_inv_rows", bytes, s);
        hipLaunchKernelGGL(ntt_inv_rows<4>, dim3(limbs), dim3(256), 0, s, c->d_tw_inv, c->d_mod, map, in, out,
                           io.in_poly_stride, io.out_poly_stride); }
        { ProfScope ps("ntt_inv_cols", bytes, s);
        hipLaunchKernelGGL(ntt_inv_cols<4>, dim3(limbs), dim3(256), 0, s, c->d_tw_inv, c->d_mod, c->d_ninv, map, out,
                           io.out_poly_stride); }
    }
}

}  // namespace ks
