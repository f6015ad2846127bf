// Device-side modular arithmetic on 64-bit residues for gfx950.
//
// There is no 64x64 multiplier on CDNA: a 64-bit high product costs four
// 32x32 multiply-adds.  Constants (twiddles, conversion factors) therefore use
// Shoup's precomputed-quotient product (one high product + two low products),
// data x data products accumulate in 128 bits and are reduced once (Barrett
// with floor(2^128/q)).  Primes are below 2^60 so lazy values up to 4q fit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef unsigned __int128 u128;

struct Acc128 {
    u64 lo, hi;
};

__device__ __forceinline__ u64 mulhi64(u64 a, u64 b) { return __umul64hi(a, b); }

__device__ __forceinline__ u64 csub(u64 a, u64 q) { return a >= q ? a - q : a; }

// a * w mod q in [0, 2q) for any 64-bit a, with wp = floor(w * 2^64 / q), w < q.
__device__ __forceinline__ u64 shoup_lazy(u64 a, u64 w, u64 wp, u64 q) {
    u64 h = mulhi64(a, wp);
    return a * w - h * q;
}

// canonical a * w mod q
__device__ __forceinline__ u64 shoup_mul(u64 a, u64 w, u64 wp, u64 q) { return csub(shoup_lazy(a, w, wp, q), q); }

__device__ __forceinline__ void acc_mad(Acc128& acc, u64 a, u64 b) {
    u64 lo = a * b, hi = mulhi64(a, b);
    acc.lo += lo;
    acc.hi += hi + (acc.lo < lo);
}

__device__ __forceinline__ void acc_add(Acc128& acc, u64 v) {
    acc.lo += v;
    acc.hi += (acc.lo < v);
}

// x = hi*2^64 + lo with hi < q  ->  x mod q, canonical.  (r1, r0) = floor(2^128 / q).
// The quotient estimate drops the low partial products, so it is short by at
// most 4; q < 2^60 keeps the remainder below 2^63.
__device__ __forceinline__ u64 barrett128(u64 hi, u64 lo, u64 q, u64 r1, u64 r0) {
    u64 qhat = hi * r1 + mulhi64(hi, r0) + mulhi64(lo, r1);
    u64 r = lo - qhat * q;
    u64 q2 = q << 1, q4 = q << 2;
    if (r >= q4) r -= q4;
    if (r >= q2) r -= q2;
    if (r >= q) r -= q;
    return r;
}

__device__ __forceinline__ u64 acc_reduce(const Acc128& acc, u64 q, u64 r1, u64 r0) {
    return barrett128(acc.hi, acc.lo, q, r1, r0);
}

// canonical a * b mod q for a, b < q
__device__ __forceinline__ u64 mulmod_barrett(u64 a, u64 b, u64 q, u64 r1, u64 r0) {
    return barrett128(mulhi64(a, b), a * b, q, r1, r0);
}

__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 q) { return csub(a + b, q); }
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }
__device__ __forceinline__ u64 negmod(u64 a, u64 q) { return a ? q - a : 0; }
