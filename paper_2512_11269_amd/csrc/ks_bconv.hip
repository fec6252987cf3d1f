// Fast RNS base conversion (Kernel Code Generation, "Base Conversion" kernel class).
//
// One thread owns one coefficient position: it reads the n_src source residues, forms
// y_i = [x_i (D/s_i)^-1]_{s_i} (canonical, so that the implicit lift is x + u D with 0 <= u < n_src) and then,
// for every target modulus t, accumulates y_i * (D/s_i mod t) as lazy representatives and reduces once
// (Kernel Code Generation: lazy modular reduction).  All constants are uniform per workgroup and arrive
// through scalar loads; every global access is a contiguous 512-byte segment per wavefront.
#include "ks_internal.hpp"

namespace ks {

// W: word type of in and out (64-bit, or 32-bit for moduli below 2^32; strides in words).
template <int NSRC, typename W>
__global__ __launch_bounds__(256) void bconv_kernel(const BConvPlan* __restrict__ plans, const W* __restrict__ in,
                                                    uint64_t in_ps, W* __restrict__ out, uint64_t out_ps, uint32_t N) {
    const BConvPlan& P = plans[blockIdx.y];
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    const W* ip = in + (uint64_t)blockIdx.z * in_ps + n;
    W* op = out + (uint64_t)blockIdx.z * out_ps + n;
    const int n_src = (int)P.n_src;
    double y[NSRC];
#pragma unroll
    for (int i = 0; i < NSRC; ++i) {
        y[i] = 0.0;
        if (i < n_src) {
            const Mod mi = P.src_mod[i];
            const double x = word_to_f64<W>(ip[(uint64_t)P.src_limb[i] * N]);
            y[i] = canon(mulmod_lazy(x, P.src_inv[i], mi), mi);
        }
    }
    const int n_dst = (int)P.n_dst;
    for (int t = 0; t < n_dst; ++t) {
        const Mod mt = P.dst_mod[t];
        double s0 = 0.0, s1 = 0.0, s2 = 0.0;  // exact partial sums against the 12-bit pieces of the factors
#pragma unroll
        for (int i = 0; i < NSRC; ++i) {
            if (i < n_src) {
                s0 = __builtin_fma(y[i], P.hat3[t][i][0], s0);
                s1 = __builtin_fma(y[i], P.hat3[t][i][1], s1);
                s2 = __builtin_fma(y[i], P.hat3[t][i][2], s2);
            }
        }
        op[(uint64_t)P.dst_limb[t] * N] = f64_to_word<W>(canon(combine3_lazy(s0, s1, s2, mt), mt));
    }
}

void launch_bconv(const ks_ctx* c, const PlanSet& plans, uint32_t limbs_moved_per_poly, const void* in, uint64_t in_ps,
                  void* out, uint64_t out_ps, uint32_t n_polys, hipStream_t s, bool words32) {
    if (n_polys == 0 || plans.n_plans == 0) return;
    const dim3 grid(c->N / 256, plans.n_plans, n_polys), block(256);
    const BConvPlan* d_plans = plans.d_plans;
    ProfScope ps(words32 ? "bconv_u32" : "bconv", (double)limbs_moved_per_poly * n_polys * c->N * (words32 ? 4.0 : 8.0), s);
#define KS_LAUNCH_BCONV(NS)                                                                                                    \
    if (words32)                                                                                                               \
        hipLaunchKernelGGL((bconv_kernel<NS, uint32_t>), grid, block, 0, s, d_plans, static_cast<const uint32_t*>(in), in_ps,  \
                           static_cast<uint32_t*>(out), out_ps, c->N);                                                        \
    else                                                                                                                       \
        hipLaunchKernelGGL((bconv_kernel<NS, uint64_t>), grid, block, 0, s, d_plans, static_cast<const uint64_t*>(in), in_ps,  \
                           static_cast<uint64_t*>(out), out_ps, c->N)
    if (plans.shape_src <= 4) KS_LAUNCH_BCONV(4);
    else if (plans.shape_src <= 8) KS_LAUNCH_BCONV(8);
    else if (plans.shape_src <= 12) KS_LAUNCH_BCONV(12);
    else KS_LAUNCH_BCONV(16);
#undef KS_LAUNCH_BCONV
}

}  // namespace ks
