// Slot-wise kernels (Kernel Code Generation, "Elementwise" kernel class): inner product with the
// evaluation key through the evaluation-domain automorphism (a gather), tensor product, and a scaled add.  These are bandwidth-bound: one thread per slot, contiguous
// 512-byte segments per wavefront, operands shared by both key components are read once ("load reuse").
#include "ks_internal.hpp"
#include "ks_tiles.hpp"

namespace ks {

constexpr int kBatchGroup = 8;  // batch items sharing one read of the key slots

template <bool GATHER>
__global__ __launch_bounds__(256) void inner_product_kernel(const Mod* __restrict__ mods, DigitRanges dg, uint32_t ell, uint32_t E,
                                                            uint32_t L, uint32_t M, uint32_t logN, const uint64_t* __restrict__ d,
                                                            uint64_t d_ps, const uint64_t* __restrict__ lifted,
                                                            const uint64_t* __restrict__ evk, uint64_t* __restrict__ acc,
                                                            uint32_t batch, uint32_t galois) {
    const uint32_t N = 1u << logN;
    const uint32_t pos = blockIdx.y;
    const uint32_t mid = pos < ell ? pos : L + (pos - ell);
    const Mod m = mods[mid];
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    const uint32_t sn = GATHER ? galois_source_slot(n, galois, logN) : n;
    double k0[kMaxDigits], k1[kMaxDigits];
#pragma unroll
    for (int j = 0; j < kMaxDigits; ++j) {
        k0[j] = k1[j] = 0.0;
        if (j < (int)dg.ndig) {
            k0[j] = u64_to_f64(evk[((uint64_t)(j * 2 + 0) * M + mid) * N + n]);
            k1[j] = u64_to_f64(evk[((uint64_t)(j * 2 + 1) * M + mid) * N + n]);
        }
    }
    const uint32_t b_lo = blockIdx.z * kBatchGroup;
    const uint32_t b_hi = min(b_lo + kBatchGroup, batch);
    for (uint32_t b = b_lo; b < b_hi; ++b) {
        double a0 = 0.0, a1 = 0.0;
#pragma unroll
        for (int j = 0; j < kMaxDigits; ++j) {
            if (j < (int)dg.ndig) {
                const bool own = pos >= dg.lo[j] && pos < dg.hi[j];
                const uint64_t* src = own ? d + (uint64_t)b * d_ps + (uint64_t)pos * N
                                          : lifted + (((uint64_t)b * dg.ndig + j) * E + pos) * N;
                const double x = u64_to_f64(src[sn]);
                a0 += mulmod_lazy(x, k0[j], m);
                a1 += mulmod_lazy(x, k1[j], m);
            }
        }
        acc[(((uint64_t)b * 2 + 0) * E + pos) * N + n] = f64_to_u64(canon(reduce_lazy(a0, m), m));
        acc[(((uint64_t)b * 2 + 1) * E + pos) * N + n] = f64_to_u64(canon(reduce_lazy(a1, m), m));
    }
}

void launch_inner_product(const ks_ctx* c, const Level& lv, const uint64_t* d, uint64_t d_ps, const uint64_t* lifted,
                          const uint64_t* evk, uint64_t* acc, uint32_t batch, uint32_t galois, hipStream_t s) {
    if (batch == 0) return;
    DigitRanges dg;
    dg.ndig = lv.ndig;
    for (uint32_t j = 0; j < kMaxDigits; ++j) {
        dg.lo[j] = j < lv.ndig ? lv.digit_lo[j] : 0;
        dg.hi[j] = j < lv.ndig ? lv.digit_hi[j] : 0;
    }
    const dim3 grid(c->N / 256, lv.E, (batch + kBatchGroup - 1) / kBatchGroup), block(256);
    // reads: every raised digit limb per ciphertext, the key once; writes: both accumulators
    ProfScope ps("inner_product", ((double)batch * (lv.ndig + 2) * lv.E + 2.0 * lv.ndig * lv.E) * c->N * 8.0, s);
    if (galois == 1)
        hipLaunchKernelGGL(inner_product_kernel<false>, grid, block, 0, s, c->d_mod, dg, lv.ell, lv.E, c->L, c->M, c->logN, d,
                           d_ps, lifted, evk, acc, batch, galois);
    else
        hipLaunchKernelGGL(inner_product_kernel<true>, grid, block, 0, s, c->d_mod, dg, lv.ell, lv.E, c->L, c->M, c->logN, d,
                           d_ps, lifted, evk, acc, batch, galois);
}

// Rotate-multiply-accumulate on the extended basis (inner sum of a baby-step giant-step transform with the division by P
// deferred to the whole sum).  One thread owns one slot of one limb position for a group of ciphertexts and walks the
// rotations: key slots and the plaintext slot of a rotation are read once per group, the raised digits and c0 come
// through the sigma_g gather, and the two running sums stay in registers until every rotation of the launch is in.
__global__ __launch_bounds__(256) void rotate_mac_kernel(const Mod* __restrict__ mods, const double* __restrict__ Pmod, DigitRanges dg,
                                                         uint32_t ell, uint32_t E, uint32_t L, uint32_t M, uint32_t logN,
                                                         const uint64_t* __restrict__ ct, uint64_t ct_bs,
                                                         const uint64_t* __restrict__ lifted, MacRotations rot,
                                                         uint64_t* __restrict__ u, uint32_t batch, int accumulate) {
    const uint32_t N = 1u << logN;
    const uint32_t pos = blockIdx.y;
    const uint32_t mid = pos < ell ? pos : L + (pos - ell);
    const Mod m = mods[mid];
    const double pm = pos < ell ? Pmod[pos] : 0.0;
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    const uint32_t b_lo = blockIdx.z * kBatchGroup;
    const uint32_t nb = min((uint32_t)kBatchGroup, batch - b_lo);
    double u0[kBatchGroup], u1[kBatchGroup];
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        u0[bi] = u1[bi] = 0.0;
        if (accumulate && bi < (int)nb) {
            u0[bi] = u64_to_f64(u[(((uint64_t)(b_lo + bi) * 2 + 0) * E + pos) * N + n]);
            u1[bi] = u64_to_f64(u[(((uint64_t)(b_lo + bi) * 2 + 1) * E + pos) * N + n]);
        }
    }
#pragma unroll 1
    for (uint32_t r = 0; r < rot.n; ++r) {
        const uint32_t sn = galois_source_slot(n, rot.galois[r], logN);
        const uint64_t* key = rot.key[r];
        double k0[kMaxDigits], k1[kMaxDigits];
#pragma unroll
        for (int j = 0; j < kMaxDigits; ++j) {
            k0[j] = k1[j] = 0.0;
            if (j < (int)dg.ndig) {
                k0[j] = u64_to_f64(key[((uint64_t)(j * 2 + 0) * M + mid) * N + n]);
                k1[j] = u64_to_f64(key[((uint64_t)(j * 2 + 1) * M + mid) * N + n]);
            }
        }
        const double w = u64_to_f64(rot.pt[r][(uint64_t)mid * N + n]);
#pragma unroll
        for (int bi = 0; bi < kBatchGroup; ++bi) {
            if (bi < (int)nb) {
                const uint64_t* cb = ct + (uint64_t)(b_lo + bi) * ct_bs;
                double t0 = 0.0, t1 = 0.0;
#pragma unroll
                for (int j = 0; j < kMaxDigits; ++j) {
                    if (j < (int)dg.ndig) {
                        const bool own = pos >= dg.lo[j] && pos < dg.hi[j];
                        const uint64_t* src = own ? cb + ((uint64_t)ell + pos) * N
                                                  : lifted + (((uint64_t)(b_lo + bi) * dg.ndig + j) * E + pos) * N;
                        const double x = u64_to_f64(src[sn]);
                        t0 += mulmod_lazy(x, k0[j], m);
                        t1 += mulmod_lazy(x, k1[j], m);
                    }
                }
                if (pos < ell) t0 += mulmod_lazy(u64_to_f64(cb[(uint64_t)pos * N + sn]), pm, m);
                // |t| <= (digits + 1) * 0.51 p, far inside the range of a lazy product; the sums grow by 0.51 p a rotation
                u0[bi] += mulmod_lazy(t0, w, m);
                u1[bi] += mulmod_lazy(t1, w, m);
            }
        }
    }
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        if (bi < (int)nb) {
            u[(((uint64_t)(b_lo + bi) * 2 + 0) * E + pos) * N + n] = f64_to_u64(canon(reduce_lazy(u0[bi], m), m));
            u[(((uint64_t)(b_lo + bi) * 2 + 1) * E + pos) * N + n] = f64_to_u64(canon(reduce_lazy(u1[bi], m), m));
        }
    }
}

void launch_rotate_mac(const ks_ctx* c, const Level& lv, const uint64_t* ct, uint64_t ct_bs, const uint64_t* lifted,
                       const MacRotations& rot, uint64_t* u, uint32_t batch, bool accumulate, hipStream_t s) {
    if (batch == 0 || rot.n == 0) return;
    DigitRanges dg;
    dg.ndig = lv.ndig;
    for (uint32_t j = 0; j < kMaxDigits; ++j) {
        dg.lo[j] = j < lv.ndig ? lv.digit_lo[j] : 0;
        dg.hi[j] = j < lv.ndig ? lv.digit_hi[j] : 0;
    }
    const uint32_t groups = (batch + kBatchGroup - 1) / kBatchGroup;
    const dim3 grid(c->N / 256, lv.E, groups), block(256);
    // per rotation: every raised digit limb and c0 per ciphertext, key and plaintext once per group; both sums written once
    const double reads = (double)rot.n * ((double)batch * (lv.ndig * lv.E + lv.ell) + (double)groups * (2.0 * lv.ndig + 1.0) * lv.E);
    ProfScope ps("rotate_mac", (reads + (double)batch * 2 * lv.E * (accumulate ? 2 : 1)) * c->N * 8.0, s);
    hipLaunchKernelGGL(rotate_mac_kernel, grid, block, 0, s, c->d_mod, c->d_Pmod, dg, lv.ell, lv.E, c->L, c->M, c->logN, ct, ct_bs, lifted,
                       rot, u, batch, accumulate ? 1 : 0);
}

// (b1, a1) x (b2, a2) -> d0 = b1 b2, d1 = a1 b2 + a2 b1, d2 = a1 a2
__global__ __launch_bounds__(256) void tensor_product_kernel(const Mod* __restrict__ mods, uint32_t ell, uint32_t N,
                                                             const uint64_t* __restrict__ cta, const uint64_t* __restrict__ ctb,
                                                             uint64_t* __restrict__ td) {
    const uint32_t i = blockIdx.y, b = blockIdx.z;
    const Mod m = mods[i];
    const uint64_t n = blockIdx.x * 256 + threadIdx.x;
    const uint64_t ct_off = ((uint64_t)b * 2 * ell + i) * N + n, comp = (uint64_t)ell * N;
    const double b1 = u64_to_f64(cta[ct_off]), a1 = u64_to_f64(cta[ct_off + comp]);
    const double b2 = u64_to_f64(ctb[ct_off]), a2 = u64_to_f64(ctb[ct_off + comp]);
    const uint64_t o = ((uint64_t)b * 3 * ell + i) * N + n;
    td[o] = f64_to_u64(canon(mulmod_lazy(b1, b2, m), m));
    td[o + comp] = f64_to_u64(canon(reduce_lazy(mulmod_lazy(a1, b2, m) + mulmod_lazy(a2, b1, m), m), m));
    td[o + 2 * comp] = f64_to_u64(canon(mulmod_lazy(a1, a2, m), m));
}

void launch_tensor_product(const ks_ctx* c, const uint64_t* cta, const uint64_t* ctb, uint64_t* td, uint32_t ell,
                           uint32_t batch, hipStream_t s) {
    if (batch == 0) return;
    ProfScope ps("tensor_product", (double)batch * ell * 7 * c->N * 8.0, s);
    hipLaunchKernelGGL(tensor_product_kernel, dim3(c->N / 256, ell, batch), dim3(256), 0, s, c->d_mod, ell, c->N, cta, ctb, td);
}

// acc[b][comp][limb] = (acc + mul * addend[b][comp][limb]) mod q_limb, canonical: the one ciphertext limb that joins the
// special limbs as a conversion source when ModDown and rescale are merged.
__global__ __launch_bounds__(256) void add_scaled_limb_kernel(const Mod* __restrict__ mods, uint32_t limb, double mul, uint32_t N,
                                                              uint64_t* __restrict__ acc, uint64_t acc_ps,
                                                              const uint64_t* __restrict__ addend, uint64_t addend_bs,
                                                              uint64_t addend_cs) {
    const Mod m = mods[limb];
    const uint32_t b = blockIdx.z >> 1, comp = blockIdx.z & 1;
    const uint64_t n = blockIdx.x * 256 + threadIdx.x;
    uint64_t* a = acc + (uint64_t)blockIdx.z * acc_ps + (uint64_t)limb * N + n;
    const double d = u64_to_f64(addend[(uint64_t)b * addend_bs + comp * addend_cs + (uint64_t)limb * N + n]);
    *a = f64_to_u64(canon(reduce_lazy(u64_to_f64(*a) + mulmod_lazy(d, mul, m), m), m));
}

void launch_add_scaled_limb(const ks_ctx* c, uint64_t* acc, uint64_t acc_ps, const uint64_t* addend, uint64_t addend_bs,
                            uint64_t addend_comp_stride, uint32_t limb, double mul, uint32_t batch, hipStream_t s) {
    if (batch == 0) return;
    ProfScope ps("add_scaled_limb", (double)batch * 2 * 3 * c->N * 8.0, s);
    hipLaunchKernelGGL(add_scaled_limb_kernel, dim3(c->N / 256, 1, batch * 2), dim3(256), 0, s, c->d_mod, limb, mul, c->N, acc, acc_ps,
                       addend, addend_bs, addend_comp_stride);
}

}  // namespace ks
