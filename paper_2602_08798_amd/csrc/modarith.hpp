// Modular arithmetic for primes below 2^50, carried in FP64 registers.
//
// Every residue is an integer-valued double.  A product a*b mod p is taken
// with the error-free transformation h = fl(a*b), l = fma(a,b,-h) and a
// quotient estimate c = rint(h * (1/p)); h - c*p and the final sum with l are
// integers below 2^53 in magnitude, so both are exact.  CDNA4 issues FP64 FMA
// at full rate while 32-bit integer multiplies run at quarter rate, which is
// why the hot kernels do not use the classic 64-bit Barrett/Montgomery
// sequence (kept below, integer-only, for the side-by-side micro-benchmark).
//
// "Lazy" values: a value known to satisfy |x| <= beta*p is carried without
// reduction as long as beta*p stays below 2^53 (beta <= 8 for p < 2^50).
// mulmod(a, b) with |a| <= A p, |b| <= B p returns r = a*b (mod p) with
// |r| <= (1/2 + 3AB/8) p; red(x) returns r = x (mod p), |r| <= (1/2 + 2^-40) p.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define CG_HD __host__ __device__ __forceinline__
#else
#define CG_HD inline
#endif

namespace cg {

struct ModD {
    double p;  // the prime
    double u;  // fl(1/p)
};

CG_HD double mulmod(double a, double b, const ModD m)
{
    const double h = a * b;
    const double l = __builtin_fma(a, b, -h);
    const double c = __builtin_rint(h * m.u);
    const double d = __builtin_fma(-c, m.p, h);
    return d + l;
}

// x (mod p), centred: |result| <= p/2 (+ rounding slack)
CG_HD double red(double x, const ModD m)
{
    const double c = __builtin_rint(x * m.u);
    return __builtin_fma(-c, m.p, x);
}

// canonical representative in [0, p) of a lazy value
CG_HD double canon(double x, const ModD m)
{
    const double r = red(x, m);
    return r < 0.0 ? r + m.p : r;
}

// a + b for canonical a, b -> canonical
CG_HD double addmod_canon(double a, double b, const ModD m)
{
    const double s = a + b;
    return s >= m.p ? s - m.p : s;
}

// uint64 residue (< 2^52) <-> double, by exponent splicing: one integer OR and one FP add
CG_HD double u64_to_f64(uint64_t x)
{
    union { uint64_t u; double d; } v;
    v.u = x | 0x4330000000000000ull;  // 2^52 + x
    return v.d - 4503599627370496.0;
}
CG_HD uint64_t f64_to_u64(double x)  // x integer-valued in [0, 2^52)
{
    union { uint64_t u; double d; } v;
    v.d = x + 4503599627370496.0;
    return v.u & 0x000FFFFFFFFFFFFFull;
}

// ---------------------------------------------------------------------------
// Integer-only 64-bit Barrett product (32-bit multiplies underneath), q < 2^50.
// Used only by the arithmetic micro-benchmark.
// ---------------------------------------------------------------------------
struct ModI {
    uint64_t q;
    uint64_t mu;  // floor(2^100 / q)
};

CG_HD uint64_t mulhi64(uint64_t a, uint64_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (uint64_t)(((unsigned __int128)a * b) >> 64);
#endif
}

CG_HD uint64_t mulmod_barrett(uint64_t a, uint64_t b, const ModI m)
{
    const uint64_t lo = a * b;
    const uint64_t hi = mulhi64(a, b);              // a*b = hi:lo < 2^100
    const uint64_t x1 = (hi << 15) | (lo >> 49);    // floor(ab / 2^49) < 2^51
    // qhat = floor(x1 * mu / 2^51), mu < 2^51
    const uint64_t plo = x1 * m.mu;
    const uint64_t phi = mulhi64(x1, m.mu);
    const uint64_t qhat = (phi << 13) | (plo >> 51);
    uint64_t r = lo - qhat * m.q;                   // true remainder + {0,1,2} q, fits 64 bits
    if (r >= 2 * m.q) r -= 2 * m.q;
    if (r >= m.q) r -= m.q;
    return r;
}

}  // namespace cg
