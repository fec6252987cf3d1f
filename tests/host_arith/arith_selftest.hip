// Host-side check of the library's double-precision modular arithmetic (ks_device.hpp) against exact
// 128-bit integer arithmetic.  Runs entirely on the CPU; prints "OK" and exits 0 when every bound holds.
#include <stdio.h>
#include <stdlib.h>
#include <math.h>
#include <stdint.h>
#include "../../paper_2512_11269_amd/csrc/ks_device.hpp"

using namespace ks;
typedef __int128 i128;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {  // xorshift64*
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return rng_state * 0x2545F4914F6CDD1Dull;
}
static int64_t rnd_signed(int bits) { return (int64_t)(rnd() >> (64 - bits)) - ((int64_t)1 << (bits - 1)); }
static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

static int64_t mod_i128(i128 x, int64_t p) { i128 r = x % p; if (r < 0) r += p; return (int64_t)r; }

static void check_prime(uint64_t p) {
    const Mod m{(double)p, 1.0 / (double)p};
    const double lim = 0.51 * (double)p;
    // conversions
    for (int i = 0; i < 20000; ++i) {
        uint64_t x = rnd() >> 12;
        if (i < 4) x = (uint64_t[]){0, 1, p - 1, (1ull << 52) - 1}[i];
        CHECK(u64_to_f64(x) == (double)x, "u64_to_f64 %llu", (unsigned long long)x);
        CHECK(f64_to_u64((double)x) == x, "f64_to_u64 %llu", (unsigned long long)x);
    }
    // mulmod_lazy: |a| <= 2^43, 0 <= b < p (also negative b up to p in magnitude)
    for (int i = 0; i < 400000; ++i) {
        int64_t a = rnd_signed(44), b = (int64_t)(rnd() % p);
        if (i % 7 == 0) a = (i & 8) ? ((int64_t)1 << 43) : -((int64_t)1 << 43);
        if (i % 11 == 0) b = (int64_t)p - 1;
        if (i % 13 == 0) { int64_t k = rnd_signed(40); i128 t = (i128)k * p + rnd_signed(3); b = 1; a = (int64_t)t; if (a > ((int64_t)1 << 43) || a < -((int64_t)1 << 43)) a = k; }
        if (i % 17 == 0) b = -b;
        const double r = mulmod_lazy((double)a, (double)b, m);
        CHECK(r == floor(r), "mulmod not integer");
        CHECK(fabs(r) <= lim, "mulmod bound a=%lld b=%lld r=%.0f p=%llu", (long long)a, (long long)b, r, (unsigned long long)p);
        CHECK(mod_i128((i128)(int64_t)r, p) == mod_i128((i128)a * b, p), "mulmod value a=%lld b=%lld", (long long)a, (long long)b);
        const double c = canon(r, m);
        CHECK(c >= 0 && c < (double)p && (int64_t)c == mod_i128((i128)a * b, p), "canon");
    }
    // products that land exactly on / next to multiples of p and half-multiples (rounding boundaries of the quotient)
    for (int i = 0; i < 100000; ++i) {
        const int64_t b = (int64_t)(rnd() % (p - 1)) + 1;
        const int64_t q = (int64_t)(rnd() >> 24);
        i128 target = (i128)q * p + ((i & 1) ? (i128)(p / 2) : 0) + rnd_signed(3);
        int64_t a = (int64_t)(target / b);
        if (a > ((int64_t)1 << 43) || a < -((int64_t)1 << 43)) continue;
        const double r = mulmod_lazy((double)a, (double)b, m);
        CHECK(fabs(r) <= lim && mod_i128((i128)(int64_t)r, p) == mod_i128((i128)a * b, p), "mulmod boundary a=%lld b=%lld", (long long)a, (long long)b);
    }
    // reduce_lazy: any |x| < 2^53
    for (int i = 0; i < 200000; ++i) {
        int64_t x = rnd_signed(54);
        if (i % 5 == 0) x = (int64_t)((rnd() >> 40) * p) + rnd_signed(3) + ((i & 1) ? (int64_t)(p / 2) : 0);
        if (x >= ((int64_t)1 << 53) || x <= -((int64_t)1 << 53)) continue;
        const double r = reduce_lazy((double)x, m);
        CHECK(fabs(r) <= lim && mod_i128((i128)(int64_t)r, p) == mod_i128((i128)x, p), "reduce x=%lld r=%.0f", (long long)x, r);
    }
    // combine3_lazy: three exact sums below 2^52
    for (int i = 0; i < 100000; ++i) {
        const uint64_t s0 = rnd() >> 12, s1 = rnd() >> 12, s2 = rnd() >> 12;
        const double r = combine3_lazy((double)s0, (double)s1, (double)s2, m);
        const i128 exact = ((i128)s2 << 24) + ((i128)s1 << 12) + s0;
        CHECK(fabs(r) <= lim && mod_i128((i128)(int64_t)r, p) == mod_i128(exact, p), "combine3");
    }
    // split3: the pieces add up, have the stated granularity and magnitude; with the centred shifted factors, sixteen
    // sources accumulate exactly and reduce to sum y_i f_i mod p
    for (int rep = 0; rep < 20000; ++rep) {
        double acc = 0.0;
        i128 exact = 0;
        for (int i = 0; i < 16; ++i) {
            uint64_t y = rnd() >> 28;  // below 2^36
            if (rep % 9 == 0) y = (uint64_t[]){0, (1ull << 36) - 1, (1ull << 24) - 1, 1ull << 23, (1ull << 23) + (1ull << 11), p - 1, 0xFFF800800ull, 0x800800ull}[(rep / 9 + i) % 8];
            uint64_t f = rnd() % p;
            if (rep % 5 == 0) f = (i & 1) ? p / 2 : p / 2 + 1;  // largest centred magnitudes
            double y2, y1, y0;
            split3((double)y, y2, y1, y0);
            CHECK(y2 + y1 + y0 == (double)y, "split3 sum %llu", (unsigned long long)y);
            CHECK(fmod(y2, 16777216.0) == 0 && y2 >= 0 && y2 <= 68719476736.0, "split3 y2 %llu", (unsigned long long)y);
            CHECK(fmod(y1, 4096.0) == 0 && fabs(y1) <= 8388608.0, "split3 y1 %llu", (unsigned long long)y);
            CHECK(fabs(y0) <= 2048.0 && y0 == floor(y0), "split3 y0 %llu", (unsigned long long)y);
            double fk[3];
            for (int k = 0; k < 3; ++k) {
                const uint64_t s = (uint64_t)(((i128)f << (12 * k)) % p);
                fk[k] = ldexp(s > p / 2 ? -(double)(p - s) : (double)s, -12 * k);
            }
            acc = __builtin_fma(y2, fk[2], __builtin_fma(y1, fk[1], __builtin_fma(y0, fk[0], acc)));
            CHECK(acc == floor(acc) && fabs(acc) < 9007199254740992.0, "split3 accumulator not an exact integer");
            exact += (i128)y * f;
        }
        const double r = reduce_lazy(acc, m);
        CHECK(fabs(r) <= lim && mod_i128((i128)(int64_t)r, p) == mod_i128(exact, p), "split3 conversion sum");
    }
    // split2 (contexts whose moduli are all below 2^32): the two pieces add up, have the stated granularity and magnitude;
    // with the centred factors cut at 16 bits, sixteen sources accumulate exactly and reduce to sum y_i f_i mod p
    if (p < (1ull << 32)) {
        for (int rep = 0; rep < 20000; ++rep) {
            double acc = 0.0;
            i128 exact = 0;
            for (int i = 0; i < 16; ++i) {
                uint64_t y = rnd() >> 32;  // below 2^32: a residue of some other modulus of such a context
                if (rep % 9 == 0) y = (uint64_t[]){0, (1ull << 32) - 1, (1ull << 16) - 1, 1ull << 15, (1ull << 15) + 1, p - 1, 0xFFFF8000ull, 0x8000ull}[(rep / 9 + i) % 8];
                uint64_t f = rnd() % p;
                if (rep % 5 == 0) f = (i & 1) ? p / 2 : p / 2 + 1;  // largest centred magnitudes
                double y1, y0;
                split2((double)y, y1, y0);
                CHECK(y1 + y0 == (double)y, "split2 sum %llu", (unsigned long long)y);
                CHECK(fmod(y1, 65536.0) == 0 && y1 >= 0 && y1 <= 4294967296.0, "split2 y1 %llu", (unsigned long long)y);
                CHECK(fabs(y0) <= 32768.0 && y0 == floor(y0), "split2 y0 %llu", (unsigned long long)y);
                double fk[2];
                for (int k = 0; k < 2; ++k) {
                    const uint64_t s = (uint64_t)(((i128)f << (16 * k)) % p);
                    fk[k] = ldexp(s > p / 2 ? -(double)(p - s) : (double)s, -16 * k);
                }
                acc = __builtin_fma(y1, fk[1], __builtin_fma(y0, fk[0], acc));
                CHECK(acc == floor(acc) && fabs(acc) < 9007199254740992.0, "split2 accumulator not an exact integer below 2^53");
                exact += (i128)y * f;
            }
            const double r = reduce_lazy(acc, m);
            CHECK(fabs(r) <= lim && mod_i128((i128)(int64_t)r, p) == mod_i128(exact, p), "split2 conversion sum");
        }
    }
    // sixteen-point passes against exact butterflies; growth bounds
    for (int rep = 0; rep < 2000; ++rep) {
        double t[16], v[16], w[16];
        int64_t e[16];
        t[0] = 0;
        for (int k = 1; k < 16; ++k) t[k] = (double)(rnd() % p);
        for (int k = 0; k < 16; ++k) { e[k] = (rep & 1) ? (int64_t)(rnd() % p) : rnd_signed(40); v[k] = (double)e[k]; }
        double in_max = 0; for (int k = 0; k < 16; ++k) in_max = fmax(in_max, fabs(v[k]));
        // exact forward: stage u pairs k, k + (8 >> u) inside groups of 16 >> u
        int64_t x[16]; for (int k = 0; k < 16; ++k) x[k] = mod_i128(e[k], p);
        for (int u = 0; u < 4; ++u) { int half = 8 >> u; for (int g = 0; g < (1 << u); ++g) { int64_t tw = (int64_t)t[(1 << u) + g]; for (int i = 0; i < half; ++i) { int k = g * 2 * half + i; int64_t y = mod_i128((i128)x[k + half] * tw, p); int64_t a = x[k]; x[k] = mod_i128((i128)a + y, p); x[k + half] = mod_i128((i128)a - y, p); } } }
        for (int k = 0; k < 16; ++k) w[k] = v[k];
        radix16_fwd(w, t, m);
        for (int k = 0; k < 16; ++k) {
            CHECK(mod_i128((i128)(int64_t)w[k], p) == x[k], "radix16_fwd value");
            CHECK(fabs(w[k]) <= in_max + 4 * lim, "radix16_fwd growth");
        }
        // shortened passes (last 4 - U0 stages only) against the same exact butterflies
        {
            int64_t y[16];
            double z[16];
            for (int k = 0; k < 16; ++k) { y[k] = mod_i128(e[k], p); z[k] = v[k]; }
            for (int u = 2; u < 4; ++u) { int half = 8 >> u; for (int g = 0; g < (1 << u); ++g) { int64_t tw = (int64_t)t[(1 << u) + g]; for (int i = 0; i < half; ++i) { int k = g * 2 * half + i; int64_t xx = mod_i128((i128)y[k + half] * tw, p); int64_t a = y[k]; y[k] = mod_i128((i128)a + xx, p); y[k + half] = mod_i128((i128)a - xx, p); } } }
            radix16_fwd<2>(z, t, m);
            for (int k = 0; k < 16; ++k) CHECK(mod_i128((i128)(int64_t)z[k], p) == y[k], "radix16_fwd<2> value");
            for (int k = 0; k < 16; ++k) { y[k] = mod_i128(e[k], p); z[k] = v[k]; }
            for (int u = 3; u >= 1; --u) { int half = 8 >> u; for (int g = 0; g < (1 << u); ++g) { int64_t tw = (int64_t)t[(1 << u) + g]; for (int i = 0; i < half; ++i) { int k = g * 2 * half + i; int64_t a = y[k], b = y[k + half]; y[k] = mod_i128((i128)a + b, p); y[k + half] = mod_i128((i128)mod_i128((i128)a - b, p) * tw, p); } } }
            if (rep & 1) {   // canonical inputs: inside the inverse pass's input range
                radix16_inv<1>(z, t, m);
                for (int k = 0; k < 16; ++k) CHECK(mod_i128((i128)(int64_t)z[k], p) == y[k], "radix16_inv<1> value");
            }
        }
        // inverse pass needs |v| <= p
        for (int k = 0; k < 16; ++k) { e[k] = (int64_t)(rnd() % (2 * p)) - (int64_t)p; v[k] = (double)e[k]; x[k] = mod_i128(e[k], p); }
        for (int u = 3; u >= 0; --u) { int half = 8 >> u; for (int g = 0; g < (1 << u); ++g) { int64_t tw = (int64_t)t[(1 << u) + g]; for (int i = 0; i < half; ++i) { int k = g * 2 * half + i; int64_t a = x[k], b = x[k + half]; x[k] = mod_i128((i128)a + b, p); x[k + half] = mod_i128((i128)(a - b) * tw, p); } } }
        radix16_inv(v, t, m);
        for (int k = 0; k < 16; ++k) {
            CHECK(mod_i128((i128)(int64_t)v[k], p) == x[k], "radix16_inv value");
            CHECK(fabs(v[k]) <= 16.0 * (double)p, "radix16_inv growth");
        }
    }
}

int main() {
    const uint64_t primes[] = {68718428161ull /* largest, N=2^16 */, 68617633793ull /* 60th, N=2^16 */, 68719403009ull /* largest, N=2^12 */,
                               68718764033ull /* 6th, N=2^12 */, 34359754753ull /* a 35-bit prime = 1 mod 2^17 */,
                               // the rest of the admitted range: the paper's word size, the top of the 32-bit range, a tiny modulus
                               268042241ull /* largest 28-bit prime = 1 mod 2^17 */, 4293918721ull /* largest below 2^32, = 1 mod 2^17 */,
                               40961ull /* = 1 mod 2^13 */};
    for (uint64_t p : primes) check_prime(p);
    if (fails) { printf("%d checks failed\n", fails); return 1; }
    printf("OK\n");
    return 0;
}
