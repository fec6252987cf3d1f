/*
 * ks.h — C ABI of the MI355X (gfx950) CKKS hybrid key-switching library.
 *
 * The operations are the ones the paper builds its encrypted-inference kernels from
 * (Background: "RNS and Limbs", "NTT", "Evaluation Keys"; Motivation: hoisting; Kernel Code
 * Generation: the NTT, Base Conversion and Elementwise kernel classes).  The paper gives no
 * formulas; the arithmetic follows the textbook algorithms it cites and is stated with each entry
 * point below.
 *
 * General conventions
 * -------------------
 *  - Ring: Z[X]/(X^N + 1), N = 2^logN.  RNS basis: ciphertext primes q_0..q_{L-1} followed by special
 *    primes p_0..p_{K-1}; "modulus id" m in [0, L+K) indexes that concatenated list.  Every modulus is
 *    an odd prime below 2^36 with m = 1 (mod 2N).
 *  - A limb is N residues in 64-bit words, N contiguous.  The entry points whose names end in _u32 take the
 *    same tensors with one residue per 32-bit word (see "32-bit words" below).  All residues handed to the
 *    library must be canonical (in [0, modulus)); every output is canonical.
 *  - Evaluation domain order is bit-reversed: slot k of a limb holds a(psi^(2*brv(k)+1)), brv = bit
 *    reversal on logN bits, psi = the primitive 2N-th root of unity of that modulus.
 *  - Digits for hybrid key-switching are contiguous groups of alpha = ceil(L/dnum) ciphertext limbs;
 *    at level ell <= L the digits cover limbs 0..ell-1 and the last one may be short.
 *  - All data pointers ("device" below) are GPU global memory owned by the caller, 16-byte aligned.
 *    Inputs are never modified; outputs must not overlap inputs unless a call says "in place".
 *    Pointers marked "host" are ordinary host memory read before the call returns.
 *  - Every compute call is asynchronous on the given HIP stream (`stream` is a hipStream_t passed as
 *    void*; NULL = default stream), performs no device-wide synchronisation and allocates no device
 *    memory (ks_ctx_create and bconv_prepare, the set-up calls, are the exceptions).
 *  - Return value: KS_OK (0) or a negative KS_E* code; ks_strerror() describes it.  On error nothing
 *    has been launched.
 */
#ifndef KS_MI355X_H
#define KS_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ks_ctx ks_ctx; /* opaque; owns only device tables (twiddles, conversion constants) */

enum {
    KS_OK = 0,
    KS_EINVAL = -1,     /* bad argument: null / misaligned pointer, unsupported size, bad modulus ... */
    KS_EWORKSPACE = -2, /* workspace pointer null or ws_bytes too small                               */
    KS_EHIP = -3,       /* a HIP runtime call failed; see ks_last_hip_error()                          */
    KS_ENOMEM = -4,     /* host or device allocation failed while building a context                   */
    KS_ENOTPREPARED = -5 /* bconv called for a (source, target) list pair that bconv_prepare has not registered */
};

enum { /* operations for ks_workspace_bytes */
    KS_OP_KEYSWITCH = 1,
    KS_OP_ROTATE_HOISTED = 2,
    KS_OP_HMULT_RELIN_RESCALE = 3,
    KS_OP_BSGS = 4,
    KS_OP_ROTATE_HOISTED_U32 = 5, /* ks_rotate_hoisted_u32 and ks_rotate_mac_hoisted_u32 */
    KS_OP_BSGS_U32 = 6            /* ks_bsgs_linear_transform_u32 */
};

/* Build the tables for one parameter set on GPU `device`.
 *   logN  : 12 .. 16 (ring degree 4096 .. 65536).
 *   q [L] : host, ciphertext primes.   p [K] : host, special primes (NULL iff K == 0).
 *   psi   : host [L+K] primitive 2N-th roots, or NULL = the smallest positive one for each modulus.
 *   dnum  : number of digits at full level (1 <= dnum <= L); dnum is ignored by the transform and
 *           base-conversion primitives.
 * Fails with KS_EINVAL if a modulus is not a prime < 2^36 with m = 1 (mod 2N), moduli repeat, a psi is
 * not a primitive 2N-th root, L + K > 255, alpha > 16 or K > 16.  The context is immutable afterwards and
 * may be used from several host threads. */
int ks_ctx_create(ks_ctx** out, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                  const uint64_t* q, const uint64_t* p, const uint64_t* psi, int device);
int ks_ctx_destroy(ks_ctx* ctx);

/* Tuning options of a context (results never depend on them).
 *   KS_OPT_BCONV_KERNEL   which base-conversion kernel the pipelines (fused with the column transform) and bconv use:
 *                         1 = vector fp64 accumulation, 2 = int8 matrix cores; 0 (default) = chosen from the launch
 *                         size (the matrix cores for launches too small to fill the chip).
 *   KS_OPT_BCONV_TARGETS  target limbs per workgroup (vector kernel, 1..4) or per lane half (matrix-core kernel, 1 or 3) of
 *                         the fused conversion kernel; 0 (default) = chosen from the launch size.
 * Not thread-safe against calls in flight on the same context from other host threads.  KS_EINVAL for an unknown
 * option or a value out of range. */
enum { KS_OPT_BCONV_TARGETS = 0, KS_OPT_BCONV_KERNEL = 1, KS_OPT_COUNT_ = 2 };
int ks_ctx_set_option(ks_ctx* ctx, int option, int value);

/* Bytes of device workspace the given operation needs for `batch` ciphertexts at level `ell`
 * (n_rot is only read for KS_OP_ROTATE_HOISTED and KS_OP_ROTATE_HOISTED_U32, which also serve the rotate-multiply-
 * accumulate calls; KS_OP_HMULT_RELIN_RESCALE serves all four multiplication entry points, KS_OP_KEYSWITCH both
 * key-switch word sizes).  Returns 0 for invalid arguments.  Large batches are processed in
 * internal chunks, so the result stops growing beyond a chunk. */
size_t ks_workspace_bytes(const ks_ctx* ctx, int op, uint32_t ell, uint32_t batch, uint32_t n_rot);

const char* ks_strerror(int code);
const char* ks_last_hip_error(void); /* text of the last HIP error seen by the calling thread */

/* Negacyclic number-theoretic transform (Background, "NTT"), in place.
 *   data    : device [batch][nlimbs][N].
 *   mod_ids : host [nlimbs], modulus id of each limb (the same for every batch item), nlimbs <= 192.
 * ntt_fwd: coefficient order in, bit-reversed evaluation order out:
 *          out[k] = sum_i a_i psi^((2 brv(k) + 1) i) mod m.   ntt_inv is its exact inverse. */
int ntt_fwd(const ks_ctx* ctx, uint64_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream);
int ntt_inv(const ks_ctx* ctx, uint64_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream);

/* Fast RNS base conversion (Kernel Code Generation, "Base Conversion" kernel class), coefficient-wise:
 *   y_i = [x_i (D/s_i)^-1]_{s_i},   out_t = (sum_i y_i (D/s_i)) mod t,   D = product of the source moduli,
 * i.e. the value x + u D (0 <= u < n_src) reduced modulo every target t; no correction of u.
 *   in  : device [batch][n_src][N], limb i modulo src_ids[i] (host, n_src <= 16, distinct).
 *   out : device [batch][n_dst][N], limb t modulo dst_ids[t] (host, n_dst <= 255).
 * The constant table of a (src_ids, dst_ids) pair is built by bconv_prepare (set-up time: one device allocation and a
 * synchronous copy, kept by the context); bconv itself allocates nothing, never synchronises and returns
 * KS_ENOTPREPARED for a pair that was not registered.  bconv_prepare is idempotent; it must not run concurrently with
 * other calls that use the same context. */
int bconv_prepare(ks_ctx* ctx, const uint32_t* src_ids, uint32_t n_src, const uint32_t* dst_ids, uint32_t n_dst);
int bconv(const ks_ctx* ctx, const uint64_t* in, const uint32_t* src_ids, uint32_t n_src,
          uint64_t* out, const uint32_t* dst_ids, uint32_t n_dst, uint32_t batch, void* stream);

/* Hybrid key-switching of one polynomial per batch item (Background, "Evaluation Keys"):
 *   INTT -> per-digit base conversion to all other moduli -> NTT -> inner product with the key over the
 *   digits -> INTT of the special limbs -> base conversion P -> q -> NTT -> (acc - conv) P^-1.
 *   d   : device [batch][ell][N], evaluation domain, limb i modulo q_i.
 *   evk : device [dnum][2][L+K][N], evaluation domain; component 0 pairs with out component 0.  The
 *         gadget factor is part of the key; only limbs q_0..q_{ell-1} and p_* of it are read.
 *   out : device [batch][2][ell][N], evaluation domain.
 *   ws  : device workspace of at least ks_workspace_bytes(ctx, KS_OP_KEYSWITCH, ell, batch, 0) bytes;
 *         contents undefined afterwards.  1 <= ell <= L. */
int ks_keyswitch(const ks_ctx* ctx, const uint64_t* d, uint32_t ell, const uint64_t* evk, uint64_t* out,
                 uint32_t batch, void* ws, size_t ws_bytes, void* stream);

/* ks_keyswitch with the boundary tensors in 32-bit words (the paper's word size: Evaluation, "Benchmarks", a 28-bit RNS basis in
 * 32-bit words): d [batch][ell][N], evk [dnum][2][L+K][N] and out [batch][2][ell][N] hold one
 * residue per uint32_t, which halves the traffic of the key, the largest tensor of the operation.  Arithmetic, workspace
 * (KS_OP_KEYSWITCH, 8-byte elements inside) and results are those of ks_keyswitch.  KS_EINVAL unless every modulus
 * of the context is below 2^32. */
int ks_keyswitch_u32(const ks_ctx* ctx, const uint32_t* d, uint32_t ell, const uint32_t* evk, uint32_t* out,
                     uint32_t batch, void* ws, size_t ws_bytes, void* stream);

/* ks_keyswitch for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a library-owned static device
 * array of KS_STATIC_WORKSPACE_BYTES (sized for one ciphertext at N = 2^16, L = 24, K = 8, dnum = 3; every GPU a
 * context has been created on holds it until the process ends).  Arguments, layouts and results as ks_keyswitch.
 * KS_EWORKSPACE if ks_workspace_bytes(ctx, KS_OP_KEYSWITCH, ell, batch, 0) exceeds that size (nothing is launched).
 * The call allocates nothing and does not synchronise.  All calls on one GPU share the one array: calls whose
 * execution may overlap on a GPU (different streams, different host threads) race on it and must be serialised
 * by the caller; calls on one stream are safe.  Nothing in the array needs clearing between calls. */
#define KS_STATIC_WORKSPACE_BYTES ((size_t)262 * 65536 * 8)
size_t ks_static_workspace_bytes(void);
int ks_keyswitch_static(const ks_ctx* ctx, const uint64_t* d, uint32_t ell, const uint64_t* evk, uint64_t* out,
                        uint32_t batch, void* stream);

/* Hoisted rotations (Motivation: hoisting): for every ciphertext the decompose-and-raise of c1 is done once
 * and shared by all n_rot Galois elements.  For each g: sigma_g (X -> X^g) is applied to the raised digits,
 * then inner product with that rotation's key, division by P, and sigma_g(c0) is added to component 0.
 *   ct       : device [batch][2][ell][N] (component 0 = c0, 1 = c1), evaluation domain.
 *   galois   : host [n_rot], odd, 0 < g < 2N.
 *   rot_keys : host array [n_rot] of device pointers, each laid out like evk above.
 *   out      : device [batch][n_rot][2][ell][N]. */
int ks_rotate_hoisted(const ks_ctx* ctx, const uint64_t* ct, uint32_t ell, const uint32_t* galois,
                      const uint64_t* const* rot_keys, uint32_t n_rot, uint64_t* out, uint32_t batch,
                      void* ws, size_t ws_bytes, void* stream);

/* Inner sum of a baby-step giant-step linear transform with the rotations kept on the extended basis ("double
 * hoisting"; DSL, matrix multiplication example: the form in which BSGS products consume hoisted rotations):
 *     out = sum_r pt_r * rot_{g_r}(ct),   one decompose-and-raise for all rotations and ONE division by P for the sum.
 * Per rotation the permuted raised digits of c1 are multiplied with that rotation's key (both accumulators, all
 * ell + K limbs), P sigma_{g_r}(c0) joins component 0, the pair is multiplied slot-wise by the plaintext pt_r and
 * added to the running sum; the sum is divided by P like a key-switch result.  With one rotation and pt = 1 the
 * result equals ks_rotate_hoisted's bit for bit.
 *   ct       : device [batch][2][ell][N], evaluation domain.
 *   galois   : host [n_rot], odd, 0 < g < 2N.       rot_keys : host [n_rot] device pointers, laid out like evk.
 *   pts      : host [n_rot] device pointers, each [L+K][N]: the plaintext reduced modulo every q_i and p_k,
 *              evaluation domain (only limbs i < ell and the special ones are read).
 *   out      : device [batch][2][ell][N].           Workspace: KS_OP_ROTATE_HOISTED.  Errors as ks_rotate_hoisted.
 * A Galois element 1 stands for the unrotated ciphertext: its term is P (c0, c1), no key is read (rot_keys[r] may be
 * NULL) and no key-switching noise is added -- unlike ks_rotate_hoisted, where g = 1 is an ordinary key-switch.  A NULL
 * plaintext pointer is the constant 1. */
int ks_rotate_mac_hoisted(const ks_ctx* ctx, const uint64_t* ct, uint32_t ell, const uint32_t* galois,
                          const uint64_t* const* rot_keys, const uint64_t* const* pts, uint32_t n_rot, uint64_t* out,
                          uint32_t batch, void* ws, size_t ws_bytes, void* stream);

/* Baby-step giant-step linear transform (DSL, matrix multiplication example), double-hoisted at both levels:
 *     out = sum_g rot_{G_g}( sum_b pts[g * n1 + b] * rot_{B_b}(ct) ).
 * Inner sums as ks_rotate_mac_hoisted with the n1 baby-step elements B_b (one decompose-and-raise of c1 serves every
 * baby step of every giant step; one division by P per giant step).  Outer sum: each inner result is raised again,
 * rotated by its giant-step element G_g on the extended basis and added to a running sum that is divided by P once.
 * n1 n2 + n2 key-switch inner products, but only n2 + 1 divisions by P and n2 + 1 decompose-and-raise steps.
 *   baby_galois [n1], giant_galois [n2] : host, odd, < 2N; 1 = no rotation (its key pointer may be NULL).
 *   baby_keys [n1], giant_keys [n2]     : host arrays of device pointers, laid out like evk.
 *   pts [n2 * n1]                       : host array of device pointers, each [L+K][N] as in ks_rotate_mac_hoisted, or
 *                                         NULL for the constant 1.
 *   ct, out : device [batch][2][ell][N].   Workspace: KS_OP_BSGS (n_rot ignored). */
int ks_bsgs_linear_transform(const ks_ctx* ctx, const uint64_t* ct, uint32_t ell, const uint32_t* baby_galois,
                             const uint64_t* const* baby_keys, uint32_t n1, const uint32_t* giant_galois,
                             const uint64_t* const* giant_keys, uint32_t n2, const uint64_t* const* pts, uint64_t* out,
                             uint32_t batch, void* ws, size_t ws_bytes, void* stream);

/* Homomorphic multiplication with relinearisation and rescale: tensor product
 * (d0, d1, d2) = (b1 b2, a1 b2 + a2 b1, a1 a2), key-switch d2 with rlk, add to (d0, d1), then drop limb
 * q_{ell-1} from both components with rounding to nearest (subtract the centred remainder, divide).
 *   cta, ctb : device [batch][2][ell][N] (component 0 = b, 1 = a), evaluation domain.  2 <= ell <= L.
 *   rlk      : device, laid out like evk.      out : device [batch][2][ell-1][N]. */
int hmult_relin_rescale(const ks_ctx* ctx, const uint64_t* cta, const uint64_t* ctb, uint32_t ell,
                        const uint64_t* rlk, uint64_t* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream);

/* The same multiplication with the key-switch's division by P and the rescale merged into one division by
 * P q_{ell-1} (Compiler, polynomial-level optimisations: "mod down merging"): P (d0, d1) is added to the
 * accumulated inner products on the ciphertext limbs, limb ell-1 joins the K special limbs as a source of one base
 * conversion to q_0..q_{ell-2}, and the result is multiplied by (P q_{ell-1})^-1.  It saves the rescale's own
 * transforms; every coefficient of the result is floor(x / (P q_{ell-1})) - u with 0 <= u <= K where
 * hmult_relin_rescale floors the first division and rounds the second, so the two differ in the low bits (same
 * noise order) and each has its own reference result.
 *   Arguments, layouts, workspace (KS_OP_HMULT_RELIN_RESCALE) and errors as hmult_relin_rescale; additionally
 *   KS_EINVAL when K + 1 exceeds the 16 sources one conversion takes. */
int hmult_relin_rescale_merged(const ks_ctx* ctx, const uint64_t* cta, const uint64_t* ctb, uint32_t ell,
                               const uint64_t* rlk, uint64_t* out, uint32_t batch, void* ws, size_t ws_bytes,
                               void* stream);

/* 32-bit words (Evaluation, "Benchmarks": the paper's parameter sets use a 28-bit RNS basis held in 32-bit words).
 * Each call below is the entry point of the same name without the suffix with every DEVICE tensor of residues --
 * ciphertexts, keys, plaintexts, results; for the transforms and the conversion the data itself -- holding one
 * residue per uint32_t in the same layout.  Arithmetic and results are identical; the traffic of those tensors
 * halves.  Intermediate values in the workspace stay 8 bytes wide, except that the rotation calls also keep the finished
 * raised digits as 32-bit words (their kernels are bound by re-reading them; the 64-bit rotation calls keep them as a
 * 32-bit word plus a byte).  Every call returns KS_EINVAL unless every modulus
 * of the context is below 2^32.  Workspace: the operation code of the 64-bit call, except that the two rotation calls
 * take KS_OP_ROTATE_HOISTED_U32 and the BSGS transform KS_OP_BSGS_U32 (the room their 32-bit raised digits take).
 *   ntt_fwd_u32 / ntt_inv_u32 : in place on [batch][nlimbs][N] uint32_t.
 *   bconv_u32                 : pairs registered with bconv_prepare serve both word sizes. */
int ntt_fwd_u32(const ks_ctx* ctx, uint32_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream);
int ntt_inv_u32(const ks_ctx* ctx, uint32_t* data, const uint32_t* mod_ids, uint32_t nlimbs, uint32_t batch, void* stream);
int bconv_u32(const ks_ctx* ctx, const uint32_t* in, const uint32_t* src_ids, uint32_t n_src,
              uint32_t* out, const uint32_t* dst_ids, uint32_t n_dst, uint32_t batch, void* stream);
int ks_rotate_hoisted_u32(const ks_ctx* ctx, const uint32_t* ct, uint32_t ell, const uint32_t* galois,
                          const uint32_t* const* rot_keys, uint32_t n_rot, uint32_t* out, uint32_t batch,
                          void* ws, size_t ws_bytes, void* stream);
int ks_rotate_mac_hoisted_u32(const ks_ctx* ctx, const uint32_t* ct, uint32_t ell, const uint32_t* galois,
                              const uint32_t* const* rot_keys, const uint32_t* const* pts, uint32_t n_rot,
                              uint32_t* out, uint32_t batch, void* ws, size_t ws_bytes, void* stream);
int ks_bsgs_linear_transform_u32(const ks_ctx* ctx, const uint32_t* ct, uint32_t ell, const uint32_t* baby_galois,
                                 const uint32_t* const* baby_keys, uint32_t n1, const uint32_t* giant_galois,
                                 const uint32_t* const* giant_keys, uint32_t n2, const uint32_t* const* pts, uint32_t* out,
                                 uint32_t batch, void* ws, size_t ws_bytes, void* stream);
int hmult_relin_rescale_u32(const ks_ctx* ctx, const uint32_t* cta, const uint32_t* ctb, uint32_t ell,
                            const uint32_t* rlk, uint32_t* out, uint32_t batch, void* ws, size_t ws_bytes,
                            void* stream);
int hmult_relin_rescale_merged_u32(const ks_ctx* ctx, const uint32_t* cta, const uint32_t* ctb, uint32_t ell,
                                   const uint32_t* rlk, uint32_t* out, uint32_t batch, void* ws, size_t ws_bytes,
                                   void* stream);

/* Per-kernel timing for benchmarks (the paper's evaluation characterises its NTT, base-conversion and
 * elementwise kernel classes separately; this exposes the same breakdown).  While enabled, every kernel the
 * library launches is bracketed by a pair of HIP events on its stream (this creates events, i.e. it is not
 * allocation-free, and adds small gaps between kernels: never enable it inside a timed throughput run).
 * ks_profile_enable(on) clears earlier records.  ks_profile_report waits for the recorded events and writes a
 * JSON array [{"kernel", "launches", "total_ms", "total_bytes"}...] into buf (host); total_bytes is the
 * algorithmic traffic (bytes each launch must read plus write).  KS_EINVAL if buf is too small. */
int ks_profile_enable(int on);
int ks_profile_report(char* buf, size_t buflen);

#ifdef __cplusplus
}
#endif
#endif /* KS_MI355X_H */
