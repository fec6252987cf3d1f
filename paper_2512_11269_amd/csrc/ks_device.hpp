// Device-side modular arithmetic for primes below 2^36, carried in IEEE double precision.
//
// gfx950 issues double-precision FMA at full rate while 32-bit integer multiplies run at quarter
// rate, so a 36x36 -> 72-bit modular product is an order of magnitude cheaper as a Barrett reduction
// with an FMA-based exact product than as integer multiply chains.  Every quantity below is an
// integer-valued double of magnitude < 2^53, hence exact; only the quotient estimate is approximate,
// and its error merely moves the result to another small representative of the same residue class.
//
// "Lazy" values: a residue may be held as any integer r with |r| <= 16 p congruent to the true
// value (Kernel Code Generation: lazy modular reduction); `canon` produces the canonical one.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// The arithmetic is plain IEEE double arithmetic, so it is callable from host code as well; the CPU-only test
// suite uses that to check every bound stated below against 128-bit integer arithmetic.
#define KS_HD __host__ __device__ __forceinline__

namespace ks {

struct Mod {
    double p;     // the modulus
    double pinv;  // 1/p rounded to nearest
};

constexpr double kTwo52 = 4503599627370496.0;

// Exact for x < 2^52: plant x in the mantissa of 2^52 and subtract 2^52.
KS_HD double u64_to_f64(uint64_t x) {
    return __builtin_bit_cast(double, x | 0x4330000000000000ull) - kTwo52;
}
// Exact for integer-valued 0 <= r < 2^52.
KS_HD uint64_t f64_to_u64(double r) {
    return __builtin_bit_cast(uint64_t, r + kTwo52) & 0x000FFFFFFFFFFFFFull;
}

// Residues at the library boundary are stored in 64-bit words or, for moduli below 2^32, in 32-bit words.
template <typename W>
KS_HD double word_to_f64(W x);
template <>
KS_HD double word_to_f64<uint64_t>(uint64_t x) { return u64_to_f64(x); }
template <>
KS_HD double word_to_f64<uint32_t>(uint32_t x) { return (double)x; }
template <typename W>
KS_HD W f64_to_word(double r);  // integer-valued canonical residue
template <>
KS_HD uint64_t f64_to_word<uint64_t>(double r) { return f64_to_u64(r); }
template <>
KS_HD uint32_t f64_to_word<uint32_t>(double r) { return (uint32_t)r; }

// a * b mod p as a small signed representative.
// Requires integer-valued |a| <= 2^43, |b| <= 2^36.  Returns r = a b (mod p) with |r| <= 0.51 p.
//   h + l = a b exactly (l is the rounding error of the product, recovered by one FMA);
//   q ~ a b / p; h - q p is an integer below 2^36 in magnitude, so the second FMA is exact too.
KS_HD double mulmod_lazy(double a, double b, Mod m) {
    double h = a * b;
    double l = __builtin_fma(a, b, -h);
    double q = __builtin_rint(h * m.pinv);
    double r = __builtin_fma(-q, m.p, h);
    return r + l;
}

// Any integer-valued |x| < 2^53 -> representative with |r| <= 0.51 p (the quotient estimate is off by at most one
// part in 2^51, the FMA is exact because its result is).
KS_HD double reduce_lazy(double x, Mod m) {
    double q = __builtin_rint(x * m.pinv);
    return __builtin_fma(-q, m.p, x);
}

// Split an integer-valued 0 <= y < 2^36 into y = y2 + y1 + y0 with y2 a multiple of 2^24 (0 <= y2 <= 2^36), y1 a
// multiple of 2^12 (|y1| <= 2^23) and |y0| <= 2^11, by rounding to nearest at the two granularities (adding and
// subtracting 1.5 * 2^(52 + g) rounds to a multiple of 2^g).  Six additions, no products.
// Use: with factors f_k = centred([f * 2^(12 k)]_t) * 2^(-12 k), |f_k| * 2^(12 k) <= 2^35, the sum
// y2 f_2 + y1 f_1 + y0 f_0 is an integer congruent to y f modulo t and at most 2^48 in magnitude, so up to sixteen
// such triples accumulate exactly in one double: a conversion costs three FMAs per source and target, the split is
// shared by all targets of the source, and one reduction per target finishes it.
KS_HD void split3(double y, double& y2, double& y1, double& y0) {
    constexpr double kRound24 = 0x1.8p76, kRound12 = 0x1.8p64;
    y2 = (y + kRound24) - kRound24;
    const double rem = y - y2;
    y1 = (rem + kRound12) - kRound12;
    y0 = rem - y1;
}

// The same for 0 <= y < 2^32 (contexts whose moduli are all below 2^32, i.e. every context the 32-bit-word entry points
// accept, the paper's 28-bit primes included): y = y1 + y0 with y1 a multiple of 2^16 and |y0| <= 2^15.  With
// f_k = centred([f * 2^(16 k)]_t) * 2^(-16 k), |f_k| * 2^(16 k) <= 2^31, the sum y1 f_1 + y0 f_0 is an integer congruent to
// y f modulo t and below 1.5 * 2^47 in magnitude: sixteen accumulate exactly (below 2^53), at two FMAs per source and
// target and three additions per split.
KS_HD void split2(double y, double& y1, double& y0) {
    constexpr double kRound16 = 0x1.8p68;
    y1 = (y + kRound16) - kRound16;
    y0 = y - y1;
}

// (s2 * 2^24 + s1 * 2^12 + s0) mod p as a lazy representative, for exact non-negative integer sums s_k < 2^52
// (the three partial sums of a base conversion whose factors were split into 12-bit pieces).
KS_HD double combine3_lazy(double s0, double s1, double s2, Mod m) {
    double r = reduce_lazy(s2, m);
    r = reduce_lazy(__builtin_fma(r, 4096.0, s1), m);
    return reduce_lazy(__builtin_fma(r, 4096.0, s0), m);
}

// Representative in (-p, p) -> canonical [0, p).
KS_HD double canon(double r, Mod m) { return r < 0.0 ? r + m.p : r; }

// The 15 twiddles of a 16-point register pass: t[2^u + g] = W[(base << u) + g] for local stage u = 0..3 and
// group g < 2^u, i.e. the sub-tree below heap node `base` of the per-modulus table W[k] = psi^brv(k).
// Loading them ahead of the butterflies lets their latency overlap the data loads.
KS_HD void load_twiddles16(double (&t)[16], const double* __restrict__ W, uint32_t base) {
    t[0] = 0.0;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int g = 0; g < (1 << u); ++g) t[(1 << u) + g] = W[(base << u) + g];
}

// Sixteen points, four decimation-in-time stages, in registers.  v[k] are 16 points whose mutual distances
// are 8, 4, 2, 1 times a common stride.  Growth: every stage adds at most 0.51 p to the magnitude.
// U0 > 0 runs only the local stages U0..3 (the last 4 - U0 stages: distances 8 >> U0 .. 1), for passes shorter than four
// stages; the table layout is the same.
template <int U0 = 0>
KS_HD void radix16_fwd(double (&v)[16], const double (&t)[16], Mod m) {
#pragma unroll
    for (int u = U0; u < 4; ++u) {
        const int half = 8 >> u;
#pragma unroll
        for (int g = 0; g < (1 << u); ++g) {
            const double w = t[(1 << u) + g];
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const int k = g * 2 * half + i;
                const double x = mulmod_lazy(v[k + half], w, m);
                v[k + half] = v[k] - x;
                v[k] = v[k] + x;
            }
        }
    }
}

// Inverse of radix16_fwd up to the factor 16 (decimation in frequency) with t built from Winv[k] = psi^-brv(k).
// Inputs must satisfy |v| <= p; sums double per stage, so outputs are bounded by 16 p.
template <int U0 = 0>
KS_HD void radix16_inv(double (&v)[16], const double (&t)[16], Mod m) {
#pragma unroll
    for (int u = 3; u >= U0; --u) {
        const int half = 8 >> u;
#pragma unroll
        for (int g = 0; g < (1 << u); ++g) {
            const double w = t[(1 << u) + g];
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const int k = g * 2 * half + i;
                const double x = v[k], y = v[k + half];
                v[k] = x + y;
                v[k + half] = mulmod_lazy(x - y, w, m);
            }
        }
    }
}

}  // namespace ks
