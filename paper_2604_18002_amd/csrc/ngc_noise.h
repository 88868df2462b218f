// Counter-based Gumbel noise for the eviction sample (Sec. 4.3 of the paper
// asks for i.i.d. Gumbel noise on the logits; the generator and the exact
// arithmetic below are this library's definition of it).
//
// Everything here must produce the same bits on every launch geometry and on
// any IEEE-754 machine, because the order of two perturbed keys can hinge on
// the last bit.  So: integer-only random words, and a logarithm spelled out as
// single correctly rounded double operations (no library log, no contraction:
// the translation unit that includes this header is compiled with
// -ffp-contract=off and uses __builtin_fma where a fused step is intended).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ngc {

// Philox-4x32 with 10 rounds (Salmon et al., SC'11).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The four random words of items 4*quad .. 4*quad+3 of one segment.
// counter = (quad, sequence, layer * 65536 + head selector, round), key = seed.
__device__ __forceinline__ void item_words(uint64_t seed, uint32_t round, uint32_t layer,
                                           uint32_t seq, uint32_t hsel, uint32_t quad,
                                           uint32_t out[4])
{
    philox4x32_10(quad, seq, (layer << 16) | (hsel & 0xFFFFu), round,
                  (uint32_t)seed, (uint32_t)(seed >> 32), out);
}

// log(x) for positive normal doubles:
//   x = 2^e m, m in [1,2); m > sqrt(2): m <- m/2, e <- e+1
//   f = m-1, s = f/(2+f), z = s^2
//   log m = 2s + s z (2/3 + 2/5 z + ... + 2/19 z^8)
//   log x = fma(e, ln2, log m)
__device__ __forceinline__ double defined_log(double x)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(x);
    int e = (int)((bits >> 52) & 0x7FFu) - 1023;
    double m = __longlong_as_double((long long)((bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull));
    if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
    const double f = m - 1.0;
    const double s = f / (2.0 + f);
    const double z = s * s;
    double p = 2.0 / 19.0;
    p = __builtin_fma(p, z, 2.0 / 17.0);
    p = __builtin_fma(p, z, 2.0 / 15.0);
    p = __builtin_fma(p, z, 2.0 / 13.0);
    p = __builtin_fma(p, z, 2.0 / 11.0);
    p = __builtin_fma(p, z, 2.0 / 9.0);
    p = __builtin_fma(p, z, 2.0 / 7.0);
    p = __builtin_fma(p, z, 2.0 / 5.0);
    p = __builtin_fma(p, z, 2.0 / 3.0);
    const double t = s * z;
    const double r = __builtin_fma(t, p, 2.0 * s);
    return __builtin_fma((double)e, 0.6931471805599453, r);
}

// Standard Gumbel variate from one random word; u is the centre of its 2^-32
// cell, so it is never 0 or 1.
__device__ __forceinline__ double gumbel_from_word(uint32_t r)
{
    const double u = ((double)r + 0.5) * 2.3283064365386963e-10;  // 2^-32
    const double w = -defined_log(u);
    return -defined_log(w);
}

// key = fl32(logit + tau * g); one double multiply, one double add, one
// conversion.  tau == 0 must not reach here (the key is then the logit).
__device__ __forceinline__ float perturb(float logit, float tau, uint32_t word)
{
    const double noise = (double)tau * gumbel_from_word(word);
    const double k = (double)logit + noise;
    return (float)k;
}

// Order-preserving code of an fp32 value: larger float <=> larger code,
// -0 below +0.
__device__ __forceinline__ float code_to_float(uint32_t c)   // inverse of ordered_code
{
    return __uint_as_float((c & 0x80000000u) ? (c & 0x7FFFFFFFu) : ~c);
}

__device__ __forceinline__ uint32_t ordered_code(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

}  // namespace ngc
