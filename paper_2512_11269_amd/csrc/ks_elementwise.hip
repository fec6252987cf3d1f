// Slot-wise kernels (Kernel Code Generation, "Elementwise" kernel class): inner product with the
// evaluation key through the evaluation-domain automorphism (a gather), tensor product, and a scaled add.  These are bandwidth-bound: one thread per slot, contiguous
// 512-byte segments per wavefront, operands shared by both key components are read once ("load reuse").
#include "ks_internal.hpp"
#include "ks_tiles.hpp"

namespace ks {

constexpr int kBatchGroup = 8;  // batch items sharing one read of the key slots

// What a gather reads for one (ciphertext, digit) at this limb position: a slot of the bundle [b][ndig][E][N] that holds
// the finished raised digits and, in the slots of a digit's own positions, the limbs of the polynomial itself.  PACKED:
// bits 0..31 of the residue from a 32-bit word array and the bits above from a byte array (5 bytes a residue); otherwise
// one 32-bit word.  These kernels are bound by the gather traffic (every rotation re-reads all raised digits of the
// chunk), so the bytes per residue are what sets their speed.
// A thread keeps one source per (ciphertext of its group, digit).  As pointers they would be one or two 64-bit scalars
// each, up to 48 pairs for three digits: more than the scalar register file holds beside everything else, and the spills
// made rotate_mac 201 vector registers wide.  So there is ONE pair of base pointers (the bundle slice of the thread's
// ciphertext group) and a 32-bit element offset per source; a load's address is base + 32-bit offset.
struct SrcBases {
    const char* lo;
    const uint8_t* hi;
};
template <bool PACKED>
struct SrcRaw {
    uint32_t lo, hi;
};
// e: element offset from the group's bases; below 2^30 (8 ciphertexts x 8 digits x 255 limbs x 2^16)
template <bool PACKED>
__device__ __forceinline__ SrcRaw<PACKED> src_load(const SrcBases& g, uint32_t e, uint32_t sn) {
    const uint32_t i = e + sn;
    SrcRaw<PACKED> r;
    r.lo = *reinterpret_cast<const uint32_t*>(g.lo + (i << 2));
    r.hi = PACKED ? g.hi[i] : 0u;
    return r;
}
template <bool PACKED>
__device__ __forceinline__ double src_f64(const SrcRaw<PACKED>& r) {
    return PACKED ? u64_to_f64((uint64_t)r.hi << 32 | r.lo) : (double)r.lo;
}
// The bundle slice of the ciphertext group that starts at batch item b_lo.
template <bool PACKED>
__device__ __forceinline__ SrcBases src_bases(const GatherSources& g, uint32_t ndig, uint32_t E, uint32_t N, uint32_t b_lo) {
    const uint64_t e = (uint64_t)b_lo * ndig * E * N;
    return SrcBases{reinterpret_cast<const char*>(g.lo + e), PACKED ? g.hi + e : nullptr};
}
// Offset of the sources of (ciphertext b of the group starting at b_lo, digit j) at limb position pos.
__device__ __forceinline__ uint32_t src_offset(uint32_t ndig, uint32_t E, uint32_t N, uint32_t b_lo, uint32_t b, uint32_t j,
                                               uint32_t pos) {
    return (((b - b_lo) * ndig + j) * E + pos) * N;
}

// Inner products through the sigma_g gather for a group of hoisted rotations: acc[r][b][c][pos] = sum_j sigma_{g_r}(src_j)[pos]
// key_r[j][c][pos].  One thread owns one slot of one limb position for a group of ciphertexts and walks the rotations of
// the launch, so the raised digits it gathers from are read from memory once per launch and from cache afterwards.
// Branch-free like rotate_mac_kernel below: the digit count is a template parameter and a short last group recomputes
// its last ciphertext, so every load of a rotation is issued before the first product.
// WK: word type of the keys; PACKED: format of the gathered sources (see SrcPtr).
// The special limbs of the result go to acc ([r][b][2][E][N] 64-bit words, the inverse transform reads them next), the
// ciphertext limbs to (accq_lo, accq_hi) as [r][b][2][ell][N] packed residues: they are only read back by the last
// kernel of the rotation, and written and read once per rotation they are a fifth of these two kernels' traffic.
template <int NDIG, typename WK, bool PACKED>
__global__ __launch_bounds__(256) void inner_product_kernel(const Mod* __restrict__ mods, uint32_t ell, uint32_t E,
                                                            uint32_t L, uint32_t M, uint32_t logN, GatherSources src, MacRotations rot,
                                                            uint64_t* __restrict__ acc, uint32_t* __restrict__ accq_lo,
                                                            uint8_t* __restrict__ accq_hi, uint32_t batch) {
    const uint32_t N = 1u << logN;
    const uint32_t pos = blockIdx.y;
    const uint32_t mid = pos < ell ? pos : L + (pos - ell);
    const Mod m = mods[mid];
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    const uint32_t b_lo = blockIdx.z * kBatchGroup;
    const SrcBases bases = src_bases<PACKED>(src, NDIG, E, N, b_lo);
    uint32_t srce[kBatchGroup][NDIG];
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        const uint32_t b = min(b_lo + bi, batch - 1);
#pragma unroll
        for (int j = 0; j < NDIG; ++j) srce[bi][j] = src_offset(NDIG, E, N, b_lo, b, j, pos);
    }
#pragma unroll 1
    for (uint32_t r = 0; r < rot.n; ++r) {
        const uint32_t sn = galois_source_slot(n, rot.galois[r], logN);
        const WK* key = static_cast<const WK*>(rot.key[r]) + (uint64_t)mid * N + n;
        WK kraw[NDIG][2];
        SrcRaw<PACKED> xraw[kBatchGroup][NDIG];
#pragma unroll
        for (int j = 0; j < NDIG; ++j) {
            kraw[j][0] = key[(uint64_t)(j * 2 + 0) * M * N];
            kraw[j][1] = key[(uint64_t)(j * 2 + 1) * M * N];
        }
#pragma unroll
        for (int bi = 0; bi < kBatchGroup; ++bi)
#pragma unroll
            for (int j = 0; j < NDIG; ++j) xraw[bi][j] = src_load<PACKED>(bases, srce[bi][j], sn);
        uint64_t* ar = acc + (uint64_t)r * batch * 2 * E * N;
        const uint64_t rq = (uint64_t)r * batch * 2 * ell * N;
#pragma unroll
        for (int bi = 0; bi < kBatchGroup; ++bi) {
            const uint32_t b = min(b_lo + bi, batch - 1);
            double a0 = 0.0, a1 = 0.0;
#pragma unroll
            for (int j = 0; j < NDIG; ++j) {
                const double x = src_f64<PACKED>(xraw[bi][j]);
                a0 += mulmod_lazy(x, word_to_f64<WK>(kraw[j][0]), m);
                a1 += mulmod_lazy(x, word_to_f64<WK>(kraw[j][1]), m);
            }
            const uint64_t u0 = f64_to_u64(canon(reduce_lazy(a0, m), m)), u1 = f64_to_u64(canon(reduce_lazy(a1, m), m));
            if (pos < ell) {  // uniform: ciphertext limbs go out packed, 5 bytes a residue
                const uint64_t e0 = rq + (((uint64_t)b * 2 + 0) * ell + pos) * N + n, e1 = e0 + (uint64_t)ell * N;
                accq_lo[e0] = (uint32_t)u0;
                accq_hi[e0] = (uint8_t)(u0 >> 32);
                accq_lo[e1] = (uint32_t)u1;
                accq_hi[e1] = (uint8_t)(u1 >> 32);
            } else {
                ar[(((uint64_t)b * 2 + 0) * E + pos) * N + n] = u0;
                ar[(((uint64_t)b * 2 + 1) * E + pos) * N + n] = u1;
            }
        }
    }
}

// bytes a gathered source residue takes
static double src_bytes(const GatherSources& g) { return g.hi ? 5.0 : 4.0; }

void launch_inner_product(const ks_ctx* c, const Level& lv, const GatherSources& src, const MacRotations& rot, uint64_t* acc,
                          const PackedDigits& accq, uint32_t batch, hipStream_t s, bool key_words32) {
    if (batch == 0 || rot.n == 0) return;
    const uint32_t groups = (batch + kBatchGroup - 1) / kBatchGroup;
    const dim3 grid(c->N / 256, lv.E, groups), block(256);
    // reads: every raised digit limb per ciphertext once per launch, each rotation's key once per group; writes: both
    // accumulators of every rotation
    const double wk = key_words32 ? 4.0 : 8.0;
    ProfScope ps("inner_product",
                 (src_bytes(src) * batch * lv.ndig * lv.E + (double)rot.n * (wk * 2.0 * lv.ndig * lv.E * groups + (16.0 * (lv.E - lv.ell) + 10.0 * lv.ell) * batch)) * c->N,
                 s);
#define KS_LAUNCH_IP_W(ND, WKT, PK)                                                                                                \
    hipLaunchKernelGGL((inner_product_kernel<ND, WKT, PK>), grid, block, 0, s, c->d_mod, lv.ell, lv.E, c->L, c->M, c->logN, src, \
                       rot, acc, accq.lo, accq.hi, batch)
#define KS_LAUNCH_IP(ND)                                                \
    if (!src.hi) KS_LAUNCH_IP_W(ND, uint32_t, false);                   \
    else if (key_words32) KS_LAUNCH_IP_W(ND, uint32_t, true);           \
    else KS_LAUNCH_IP_W(ND, uint64_t, true)
    switch (lv.ndig) {
        case 1: KS_LAUNCH_IP(1); break;
        case 2: KS_LAUNCH_IP(2); break;
        case 3: KS_LAUNCH_IP(3); break;
        case 4: KS_LAUNCH_IP(4); break;
        case 5: KS_LAUNCH_IP(5); break;
        case 6: KS_LAUNCH_IP(6); break;
        case 7: KS_LAUNCH_IP(7); break;
        default: KS_LAUNCH_IP(8); break;
    }
#undef KS_LAUNCH_IP
#undef KS_LAUNCH_IP_W
}

// Rotate-multiply-accumulate on the extended basis (inner sum of a baby-step giant-step transform with the division by P
// deferred to the whole sum).  One thread owns one slot of one limb position for a group of ciphertexts and walks the
// rotations: key slots and the plaintext slot of a rotation are read once per group, the raised digits and c0 come
// through the sigma_g gather, and the two running sums stay in registers until every rotation of the launch is in.
// Branch-free within a rotation on purpose (digit count as a template parameter, a short last group recomputes its last
// ciphertext, special limbs read a c0 limb they multiply by zero): every load of a rotation is then issued before the
// first product.  Galois element 1 is the unrotated ciphertext (P (c0, c1), no key read).
// WC: word type of the ciphertext ct (64-bit with packed sources, 32-bit with 32-bit sources).
template <int NDIG, typename WK, bool PACKED>
__global__ __launch_bounds__(256) void rotate_mac_kernel(const Mod* __restrict__ mods, const double* __restrict__ Pmod,
                                                         uint32_t ell, uint32_t E, uint32_t L, uint32_t M, uint32_t logN,
                                                         const void* __restrict__ ct_, uint64_t ct_bs, GatherSources src,
                                                         MacRotations rot, const uint64_t* __restrict__ one,
                                                         uint64_t* __restrict__ u, uint32_t batch, int accumulate) {
    using WC = std::conditional_t<PACKED, uint64_t, uint32_t>;
    const WC* ct = static_cast<const WC*>(ct_);
    const uint32_t N = 1u << logN;
    const uint32_t pos = blockIdx.y;
    const uint32_t mid = pos < ell ? pos : L + (pos - ell);
    const Mod m = mods[mid];
    const uint32_t c0_limb = min(pos, ell - 1);
    const double pm = pos < ell ? Pmod[c0_limb] : 0.0;
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    const uint32_t b_lo = blockIdx.z * kBatchGroup;
    const SrcBases bases = src_bases<PACKED>(src, NDIG, E, N, b_lo);
    // per ciphertext of the group: where its c0 limb and its NDIG source limbs of this position start
    const WC* c0p[kBatchGroup];
    uint32_t srce[kBatchGroup][NDIG];
    uint64_t* up[kBatchGroup];
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        const uint32_t b = min(b_lo + bi, batch - 1);
        c0p[bi] = ct + (uint64_t)b * ct_bs + (uint64_t)c0_limb * N;
#pragma unroll
        for (int j = 0; j < NDIG; ++j) srce[bi][j] = src_offset(NDIG, E, N, b_lo, b, j, pos);
        up[bi] = u + (((uint64_t)b * 2) * E + pos) * N + n;
    }
    double u0[kBatchGroup], u1[kBatchGroup];
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        u0[bi] = accumulate ? u64_to_f64(up[bi][0]) : 0.0;
        u1[bi] = accumulate ? u64_to_f64(up[bi][(uint64_t)E * N]) : 0.0;
    }
#pragma unroll 1
    for (uint32_t r = 0; r < rot.n; ++r) {
        // the plaintext slot; a null plaintext is the constant 1, read (by every lane) from a one-word table so that the
        // load stays unconditional
        // (the table holds the 64-bit word 1, whose low half is the 32-bit word 1)
        const WK* wp = rot.pt[r] ? static_cast<const WK*>(rot.pt[r]) + (uint64_t)mid * N + n : reinterpret_cast<const WK*>(one);
        if (rot.galois[r] == 1) {  // uniform: the unrotated ciphertext, P (c0, c1), no key
            WC c0raw[kBatchGroup], c1raw[kBatchGroup];
            const WK wraw = *wp;
#pragma unroll
            for (int bi = 0; bi < kBatchGroup; ++bi) {
                c0raw[bi] = c0p[bi][n];
                c1raw[bi] = c0p[bi][(uint64_t)ell * N + n];
            }
            const double pw = mulmod_lazy(pm, word_to_f64<WK>(wraw), m);
#pragma unroll
            for (int bi = 0; bi < kBatchGroup; ++bi) {
                u0[bi] += mulmod_lazy(word_to_f64<WC>(c0raw[bi]), pw, m);
                u1[bi] += mulmod_lazy(word_to_f64<WC>(c1raw[bi]), pw, m);
            }
            continue;
        }
        const uint32_t sn = galois_source_slot(n, rot.galois[r], logN);
        const WK* key = static_cast<const WK*>(rot.key[r]) + (uint64_t)mid * N + n;
        WK kraw[NDIG][2];
        SrcRaw<PACKED> xraw[kBatchGroup][NDIG];
        WC craw[kBatchGroup];
#pragma unroll
        for (int j = 0; j < NDIG; ++j) {
            kraw[j][0] = key[(uint64_t)(j * 2 + 0) * M * N];
            kraw[j][1] = key[(uint64_t)(j * 2 + 1) * M * N];
        }
        const WK wraw = *wp;
#pragma unroll
        for (int bi = 0; bi < kBatchGroup; ++bi) {
#pragma unroll
            for (int j = 0; j < NDIG; ++j) xraw[bi][j] = src_load<PACKED>(bases, srce[bi][j], sn);
            craw[bi] = c0p[bi][sn];
        }
        // the plaintext slot is folded into the key slots and into P once per rotation, not multiplied per ciphertext
        const double w = word_to_f64<WK>(wraw), pw = mulmod_lazy(pm, w, m);
        double kw[NDIG][2];
#pragma unroll
        for (int j = 0; j < NDIG; ++j) {
            kw[j][0] = mulmod_lazy(word_to_f64<WK>(kraw[j][0]), w, m);
            kw[j][1] = mulmod_lazy(word_to_f64<WK>(kraw[j][1]), w, m);
        }
#pragma unroll
        for (int bi = 0; bi < kBatchGroup; ++bi) {
            double t0 = mulmod_lazy(word_to_f64<WC>(craw[bi]), pw, m), t1 = 0.0;
#pragma unroll
            for (int j = 0; j < NDIG; ++j) {
                const double x = src_f64<PACKED>(xraw[bi][j]);
                t0 += mulmod_lazy(x, kw[j][0], m);
                t1 += mulmod_lazy(x, kw[j][1], m);
            }
            // the sums grow by at most (digits + 1) * 0.51 p a rotation: below 2^43 after the 16 rotations of a launch
            u0[bi] += t0;
            u1[bi] += t1;
        }
    }
#pragma unroll
    for (int bi = 0; bi < kBatchGroup; ++bi) {
        up[bi][0] = f64_to_u64(canon(reduce_lazy(u0[bi], m), m));
        up[bi][(uint64_t)E * N] = f64_to_u64(canon(reduce_lazy(u1[bi], m), m));
    }
}

void launch_rotate_mac(const ks_ctx* c, const Level& lv, const void* ct, uint64_t ct_bs, const GatherSources& src,
                       const MacRotations& rot, uint64_t* u, uint32_t batch, bool accumulate, hipStream_t s, bool key_words32) {
    if (batch == 0 || rot.n == 0) return;
    const uint32_t groups = (batch + kBatchGroup - 1) / kBatchGroup;
    const dim3 grid(c->N / 256, lv.E, groups), block(256);
    // Algorithmic traffic: the raised digits and c0 of a ciphertext once (the rotations of a launch re-read them through
    // the gather; those re-reads are meant to come from cache), key and plaintext of every rotation once per group, both
    // sums written once.  Algorithmic work per slot, ciphertext and rotation: 2 NDIG + 1 modular products (+ 2 NDIG + 1 per group).
    const double reads = batch * (src_bytes(src) * lv.ndig * lv.E + (src.hi ? 8.0 : 4.0) * lv.ell) +
                         (key_words32 ? 4.0 : 8.0) * (double)rot.n * groups * (2.0 * lv.ndig + 1.0) * lv.E;
    ProfScope ps("rotate_mac", (reads + (double)batch * 16 * lv.E * (accumulate ? 2 : 1)) * c->N, s,
                 (double)rot.n * batch * lv.E * c->N * (7.0 * (2 * lv.ndig + 1)));
#define KS_LAUNCH_MAC_W(ND, WKT, PK)                                                                                                  \
    hipLaunchKernelGGL((rotate_mac_kernel<ND, WKT, PK>), grid, block, 0, s, c->d_mod, c->d_Pmod, lv.ell, lv.E, c->L, c->M, c->logN, \
                       ct, ct_bs, src, rot, c->d_one, u, batch, accumulate ? 1 : 0)
#define KS_LAUNCH_MAC(ND)                                               \
    if (!src.hi) KS_LAUNCH_MAC_W(ND, uint32_t, false);                  \
    else if (key_words32) KS_LAUNCH_MAC_W(ND, uint32_t, true);          \
    else KS_LAUNCH_MAC_W(ND, uint64_t, true)
    switch (lv.ndig) {
        case 1: KS_LAUNCH_MAC(1); break;
        case 2: KS_LAUNCH_MAC(2); break;
        case 3: KS_LAUNCH_MAC(3); break;
        case 4: KS_LAUNCH_MAC(4); break;
        case 5: KS_LAUNCH_MAC(5); break;
        case 6: KS_LAUNCH_MAC(6); break;
        case 7: KS_LAUNCH_MAC(7); break;
        default: KS_LAUNCH_MAC(8); break;
    }
#undef KS_LAUNCH_MAC
#undef KS_LAUNCH_MAC_W
}

// (b1, a1) x (b2, a2) -> d0 = b1 b2, d1 = a1 b2 + a2 b1, d2 = a1 a2.  d2, the polynomial that is key-switched, goes out as
// 64-bit words ([b][ell][N]); d0 and d1 are only added back by the last kernel of the chain and go out packed
// ([b][2][ell][N]: bits 0..31 in dq_lo, the bits above in dq_hi).
template <typename W>
__global__ __launch_bounds__(256) void tensor_product_kernel(const Mod* __restrict__ mods, uint32_t ell, uint32_t N,
                                                             const W* __restrict__ cta, const W* __restrict__ ctb,
                                                             uint64_t* __restrict__ d2, uint32_t* __restrict__ dq_lo,
                                                             uint8_t* __restrict__ dq_hi) {
    const uint32_t i = blockIdx.y, b = blockIdx.z;
    const Mod m = mods[i];
    const uint64_t n = blockIdx.x * 256 + threadIdx.x;
    const uint64_t ct_off = ((uint64_t)b * 2 * ell + i) * N + n, comp = (uint64_t)ell * N;
    const double b1 = word_to_f64<W>(cta[ct_off]), a1 = word_to_f64<W>(cta[ct_off + comp]);
    const double b2 = word_to_f64<W>(ctb[ct_off]), a2 = word_to_f64<W>(ctb[ct_off + comp]);
    const uint64_t u0 = f64_to_u64(canon(mulmod_lazy(b1, b2, m), m));
    const uint64_t u1 = f64_to_u64(canon(reduce_lazy(mulmod_lazy(a1, b2, m) + mulmod_lazy(a2, b1, m), m), m));
    dq_lo[ct_off] = (uint32_t)u0;
    dq_hi[ct_off] = (uint8_t)(u0 >> 32);
    dq_lo[ct_off + comp] = (uint32_t)u1;
    dq_hi[ct_off + comp] = (uint8_t)(u1 >> 32);
    d2[((uint64_t)b * ell + i) * N + n] = f64_to_u64(canon(mulmod_lazy(a1, a2, m), m));
}

void launch_tensor_product(const ks_ctx* c, const void* cta, const void* ctb, uint64_t* d2, const PackedDigits& dq, uint32_t ell,
                           uint32_t batch, hipStream_t s, bool in_words32) {
    if (batch == 0) return;
    ProfScope ps("tensor_product", (double)batch * ell * ((in_words32 ? 16 : 32) + 8 + 10) * c->N, s);
    if (in_words32)
        hipLaunchKernelGGL(tensor_product_kernel<uint32_t>, dim3(c->N / 256, ell, batch), dim3(256), 0, s, c->d_mod, ell, c->N,
                           static_cast<const uint32_t*>(cta), static_cast<const uint32_t*>(ctb), d2, dq.lo, dq.hi);
    else
        hipLaunchKernelGGL(tensor_product_kernel<uint64_t>, dim3(c->N / 256, ell, batch), dim3(256), 0, s, c->d_mod, ell, c->N,
                           static_cast<const uint64_t*>(cta), static_cast<const uint64_t*>(ctb), d2, dq.lo, dq.hi);
}

// acc[b][comp][limb] = (acc + mul * addend[b][comp][limb]) mod q_limb, canonical: the one ciphertext limb that joins the
// special limbs as a conversion source when ModDown and rescale are merged.  The addend is packed ([b][2][ell][N]).
__global__ __launch_bounds__(256) void add_scaled_limb_kernel(const Mod* __restrict__ mods, uint32_t limb, double mul, uint32_t ell,
                                                              uint32_t N, uint64_t* __restrict__ acc, uint64_t acc_ps,
                                                              const uint32_t* __restrict__ addend_lo,
                                                              const uint8_t* __restrict__ addend_hi) {
    const Mod m = mods[limb];
    const uint64_t n = blockIdx.x * 256 + threadIdx.x;
    uint64_t* a = acc + (uint64_t)blockIdx.z * acc_ps + (uint64_t)limb * N + n;
    const uint64_t e = ((uint64_t)blockIdx.z * ell + limb) * N + n;   // blockIdx.z = 2 b + comp
    const double d = u64_to_f64((uint64_t)addend_hi[e] << 32 | addend_lo[e]);
    *a = f64_to_u64(canon(reduce_lazy(u64_to_f64(*a) + mulmod_lazy(d, mul, m), m), m));
}

void launch_add_scaled_limb(const ks_ctx* c, uint64_t* acc, uint64_t acc_ps, const PackedDigits& addend, uint32_t ell, uint32_t limb,
                            double mul, uint32_t batch, hipStream_t s) {
    if (batch == 0) return;
    ProfScope ps("add_scaled_limb", (double)batch * 2 * (16 + 5) * c->N, s);
    hipLaunchKernelGGL(add_scaled_limb_kernel, dim3(c->N / 256, 1, batch * 2), dim3(256), 0, s, c->d_mod, limb, mul, ell, c->N, acc,
                       acc_ps, addend.lo, addend.hi);
}

}  // namespace ks
