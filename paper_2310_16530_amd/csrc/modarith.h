// Device-side 64-bit modular arithmetic for primes below 2^61.
//
// Three forms are used, all exact:
//   * Shoup multiplication by a constant w with companion w' = floor(w*2^64/q):
//       x*w - floor(x*w'/2^64)*q  lies in [0, 2q) for every 64-bit x.
//   * Harvey-style lazy butterflies that keep values in [0, 4q) (forward) or
//     [0, 2q) (inverse), so that a butterfly costs one Shoup product.
//   * Montgomery reduction of a 128-bit accumulator (sum of products), which
//     returns acc * 2^-64 mod q in [0, 2q) whenever acc < q * 2^64; the factor
//     2^-64 is cancelled by keeping one operand (a constant) in Montgomery form
//     or by a second reduction with 2^128 mod q.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;

struct u128w {
    u64 lo, hi;
};

__device__ __forceinline__ u64 csub(u64 x, u64 q) { return x >= q ? x - q : x; }

__device__ __forceinline__ u64 mul_shoup_lazy(u64 x, u64 w, u64 wp, u64 q) {
    u64 h = __umul64hi(x, wp);
    return x * w - h * q;
}

__device__ __forceinline__ u64 mul_shoup(u64 x, u64 w, u64 wp, u64 q) { return csub(mul_shoup_lazy(x, w, wp, q), q); }

__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 q) { return csub(a + b, q); }
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

// acc += a*b (128-bit)
__device__ __forceinline__ void mac128(u128w& acc, u64 a, u64 b) {
    u64 lo = a * b;
    u64 hi = __umul64hi(a, b);
    acc.lo += lo;
    acc.hi += hi + (acc.lo < lo ? 1 : 0);
}

// Montgomery reduction: returns acc * 2^-64 mod q, in [0, 2q), for acc < q*2^64.
// qneg = -q^-1 mod 2^64.
__device__ __forceinline__ u64 redc_lazy(u128w acc, u64 q, u64 qneg) {
    u64 m = acc.lo * qneg;
    u64 t = __umul64hi(m, q);
    // acc.lo + (m*q).lo == 0 mod 2^64 ; carry out is 1 unless acc.lo == 0
    return acc.hi + t + (acc.lo != 0 ? 1 : 0);
}

__device__ __forceinline__ u64 redc(u128w acc, u64 q, u64 qneg) { return csub(redc_lazy(acc, q, qneg), q); }

// Full product of two canonical residues, both variable: REDC twice (the second with 2^128 mod q).
__device__ __forceinline__ u64 mulmod_var(u64 a, u64 b, u64 q, u64 qneg, u64 r2) {
    u128w p = {0, 0};
    mac128(p, a, b);
    u64 t = redc_lazy(p, q, qneg);  // a*b*2^-64, < 2q
    u128w p2 = {0, 0};
    mac128(p2, t, r2);
    return redc(p2, q, qneg);
}

// Reduce a 128-bit sum of products of canonical residues (acc < q*2^64) to its canonical residue.
__device__ __forceinline__ u64 reduce128(u128w acc, u64 q, u64 qneg, u64 r2) {
    u64 t = redc_lazy(acc, q, qneg);
    u128w p2 = {0, 0};
    mac128(p2, t, r2);
    return redc(p2, q, qneg);
}
