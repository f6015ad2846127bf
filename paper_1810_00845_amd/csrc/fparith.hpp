// Exact modular arithmetic on integers carried in fp64, for primes below 2^50.
//
// CDNA issues fp64 FMA at full rate but 32-bit integer multiplies at quarter
// rate, and a 64x64 high product needs four of those.  A residue below 2^50
// is exactly representable in a double, and the product of two of them is
// recovered exactly as h + l with h = fl(a*b), l = fma(a, b, -h).  With
// q = rint(h / p) the value h - q*p is an integer below 2^53 in magnitude, so
// fma(-q, p, h) is exact and so is adding l.  Every function here returns an
// exact integer congruent to the true result; only the range is "lazy".
//
// Ranges (kappa = p / 2^50 <= 1):
//   fp_mulmod(a, b):  |result| <= p/2 + 3 * 2^-53 * |a*b|   (needs |a|, |b| <= 2^53 exact integers)
//   fp_norm(v):       |result| <= p/2 * (1 + 2^-48)          (needs |v| <= 2^53)
// Values must stay below 2^53 in magnitude between normalisations.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FP_HD __host__ __device__ __forceinline__
#else
#define FP_HD inline
#endif

// a * b - q * p with q the integer nearest to a*b/p (up to the estimate's error)
FP_HD double fp_mulmod(double a, double b, double p, double pinv) {
    const double h = a * b;
    const double l = __builtin_fma(a, b, -h);
    const double q = __builtin_rint(h * pinv);
    const double r = __builtin_fma(-q, p, h);
    return r + l;
}

// v - rint(v/p) * p
FP_HD double fp_norm(double v, double p, double pinv) {
    const double q = __builtin_rint(v * pinv);
    return __builtin_fma(-q, p, v);
}

// non-negative integer below 2^52 -> double, by planting it in the mantissa of 2^52
FP_HD double fp_from_u64(uint64_t x) {
    union { uint64_t u; double d; } c;
    c.u = x | 0x4330000000000000ULL;
    return c.d - 4503599627370496.0;
}

// integer in [0, 2^52) held in a double -> uint64
FP_HD uint64_t fp_to_u64(double v) {
    union { uint64_t u; double d; } c;
    c.d = v + 4503599627370496.0;
    return c.u & 0x000FFFFFFFFFFFFFULL;
}

// any lazy value -> canonical residue in [0, p)
FP_HD uint64_t fp_canonical(double v, double p, double pinv) {
    double r = fp_norm(v, p, pinv);
    r = r < 0.0 ? r + p : r;
    // a tie-sized excursion (|r| = p/2 + small) still lands in [0, p)
    return fp_to_u64(r);
}

// canonical residue -> centred double in (-p/2, p/2]
FP_HD double fp_centred_from_u64(uint64_t x, double p, double half) {
    const double v = fp_from_u64(x);
    return v > half ? v - p : v;
}
