// Modular arithmetic for the key-switch kernels, in two interchangeable "arithmetic policies".
//
// IntAr  -- 64-bit integer residues, any prime below 2^61:
//   * Shoup multiplication by a constant w with companion w' = floor(w*2^64/q):
//       x*w - floor(x*w'/2^64)*q  lies in [0, 2q) for every 64-bit x.
//   * Harvey-style lazy butterflies keeping values in [0, 4q) (forward) or [0, 2q) (inverse).
//   * Montgomery reduction of a 128-bit accumulator: acc * 2^-64 mod q in [0, 2q) for acc < q*2^64.
//
// FpAr   -- residues held as integer-valued doubles (possibly negative), primes below 3*2^48.
//   On CDNA4 an FP64 FMA issues at the rate of one 32-bit integer multiply (four cycles per wave), and a Shoup
//   product of 64-bit words needs ten of those, so for the ~50-bit ciphertext primes the butterflies run on the
//   FP64 pipe.  Everything is
//   exact: for integers a, w with |a| <= A*q (A <= 8), 0 <= w < q < 3*2^48,
//       h = fl(a*w), l = fma(a, w, -h)          (a*w = h + l exactly)
//       c = rint(fl(h * fl(1/q)))               (|c - a*w/q| <= 0.5 + 3A/8)
//       r = fma(-c, q, h) + l                   (both steps exact: integers below 2^53)
//   gives r = a*w (mod q) with |r| <= (0.5 + 3A/8) q.  Four forward stages started from |x| <= q
//   stay below 7q, four inverse stages started from |x| <= q/2 stay at or below 8q < 2^53; a
//   3-instruction reduction x - rint(x/q)*q brings values back to |x| <= q/2 between rounds.
//
// All functions are __host__ __device__ so that the same source is unit-tested on the CPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;
typedef unsigned __int128 u128_t;

#define HD __host__ __device__ __forceinline__

// primes strictly below this bound use FpAr
#define CKKS_FP_PRIME_LIMIT (3ull << 48)

struct u128w {
    u64 lo, hi;
};

HD u64 mulhi64(u64 a, u64 b) { return (u64)(((u128_t)a * b) >> 64); }
HD u64 csub(u64 x, u64 q) { return x >= q ? x - q : x; }

HD u64 mul_shoup_lazy(u64 x, u64 w, u64 wp, u64 q) {
    u64 h = mulhi64(x, wp);
    return x * w - h * q;
}
HD u64 mul_shoup(u64 x, u64 w, u64 wp, u64 q) { return csub(mul_shoup_lazy(x, w, wp, q), q); }
HD u64 addmod(u64 a, u64 b, u64 q) { return csub(a + b, q); }
HD u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

HD void mac128(u128w& acc, u64 a, u64 b) {
    u128_t p = (u128_t)a * b + (((u128_t)acc.hi << 64) | acc.lo);
    acc.lo = (u64)p;
    acc.hi = (u64)(p >> 64);
}

// acc * 2^-64 mod q in [0, 2q), for acc < q*2^64.  qneg = -q^-1 mod 2^64.
HD u64 redc_lazy(u128w acc, u64 q, u64 qneg) {
    u64 m = acc.lo * qneg;
    u64 t = mulhi64(m, q);
    return acc.hi + t + (acc.lo != 0 ? 1 : 0);
}
HD u64 redc(u128w acc, u64 q, u64 qneg) { return csub(redc_lazy(acc, q, qneg), q); }

// canonical residue of a 128-bit sum of products (acc < q*2^64): REDC, then REDC against 2^128 mod q
HD u64 reduce128(u128w acc, u64 q, u64 qneg, u64 r2) {
    u64 t = redc_lazy(acc, q, qneg);
    u128w p2 = {0, 0};
    mac128(p2, t, r2);
    return redc(p2, q, qneg);
}
HD u64 mulmod_var(u64 a, u64 b, u64 q, u64 qneg, u64 r2) {
    u128w p = {0, 0};
    mac128(p, a, b);
    return reduce128(p, q, qneg, r2);
}

// Word formats of base-conversion sources (the coefficients times the conversion pre-factor that the last
// inverse stage leaves for the conversion kernels):
//   SRC_CANON  canonical integer            SRC_F64  canonical integer as a double (FpAr primes only)
//   SRC_DIGITS eight signed base-256 digits d_k in [-128, 127], y = sum d_k 256^k, digit k stored in byte k as
//              d_k + 128 with the top bit flipped, i.e. as the two's-complement byte the matrix cores read:
//              word = (y + B) ^ B with B = 0x80 in every byte (y < 2^63 - B, here y < 2^61).
enum SrcFormat { SRC_CANON = 0, SRC_F64 = 1, SRC_DIGITS = 2 };
#define CKKS_DIGIT_BIAS 0x8080808080808080ull
HD u64 digits_encode(u64 y) { return (y + CKKS_DIGIT_BIAS) ^ CKKS_DIGIT_BIAS; }
HD u64 digits_decode(u64 w) { return (w ^ CKKS_DIGIT_BIAS) - CKKS_DIGIT_BIAS; }

// ------------------------------------------------------------------ per-prime constants
struct PrimeConst {
    u64 q;        // the prime
    u64 qneg;     // -q^-1 mod 2^64
    u64 r2;       // 2^128 mod q
    u64 r1;       // 2^64 mod q
    u64 r1_p;     // its Shoup companion
    double qd;    // q as a double (exact for FpAr primes)
    double qinv;  // fl(1/q)
    u32 fp;       // 1 if the prime uses FpAr
    u32 pad;
};

// scaling constants of the last inverse-NTT stage: sx multiplies the sums, sy the differences
// (sy already includes the stage's twiddle); Shoup companions for IntAr, doubles for FpAr.
struct InvScale {
    u64 sx, sx_p, sy, sy_p;
    double sxd, syd;
};

// ------------------------------------------------------------------------------ IntAr
struct IntAr {
    typedef u64 T;
    static constexpr bool is_fp = false;

    struct Mod {
        u64 q, q2, qneg, r1, r1_p;
    };
    struct Tw {
        u64 w, wp;
    };
    static HD Mod mod(const PrimeConst& p) { return Mod{p.q, 2 * p.q, p.qneg, p.r1, p.r1_p}; }
    // tables: tw_int [prime][4][N] = fwd w, fwd w', inv w, inv w'
    static HD Tw tw(const u64* ti, const double*, u32 idx, u32 N, bool inverse) {
        const u64* b = ti + (inverse ? 2 * (size_t)N : 0);
        return Tw{b[idx], b[N + idx]};
    }
    static HD T from_canon(u64 v, const Mod&) { return v; }
    static HD T from_raw(u64 v) { return v; }
    static HD u64 to_raw(T v) { return v; }
    static HD T from_f64_lazy(double, const Mod&) { return 0; }  // FP64 conversion path is FpAr-only
    // product of two canonical residues, as a value the transforms accept
    static HD T mul_canon(u64 a, u64 b, const PrimeConst& p, const Mod&) { return mulmod_var(a, b, p.q, p.qneg, p.r2); }
    // forward: values in [0, 8q) (8q < 2^64 for primes below 2^61).  A stage adds less than 2q to its inputs
    // (the product is in [0, 2q) for any 64-bit Y), so inputs below 6q need no reduction; RED takes 4q off
    // inputs that may have reached 6q..8q first.  NttCore fixes per stage which of the two applies.
    template <bool RED>
    static HD void bfly_fwd(T& X, T& Y, const Tw& t, const Mod& m) {
        u64 x = X;
        if (RED) {
            const u64 q4 = m.q2 + m.q2;
            x = x >= q4 ? x - q4 : x;
        }
        u64 r = mul_shoup_lazy(Y, t.w, t.wp, m.q);
        X = x + r;
        Y = x - r + m.q2;
    }
    // inverse: values in [0, 2q)
    static HD void bfly_inv(T& X, T& Y, const Tw& t, const Mod& m) {
        u64 s = X + Y;
        u64 d = X - Y + m.q2;
        X = s >= m.q2 ? s - m.q2 : s;
        Y = mul_shoup_lazy(d, t.w, t.wp, m.q);
    }
    static HD T round_reduce(T v, const Mod&) { return v; }  // lazy ranges are invariants: nothing to do
    static HD u64 canon_fwd(T v, const Mod& m) { return csub(csub(csub(v, m.q2 + m.q2), m.q2), m.q); }  // from [0, 8q)
    static HD u64 canon_inv(T v, const Mod& m) { return csub(v, m.q); }
    // last inverse stage with scaling, canonical results (fmt: SRC_CANON or SRC_DIGITS; SRC_F64 does not apply)
    static HD void bfly_inv_last(T& X, T& Y, const InvScale& s, const Mod& m, u32 fmt, u64& ox, u64& oy) {
        u64 a = X + Y, d = X - Y + m.q2;
        ox = mul_shoup(a, s.sx, s.sx_p, m.q);
        oy = mul_shoup(d, s.sy, s.sy_p, m.q);
        if (fmt == SRC_DIGITS) ox = digits_encode(ox), oy = digits_encode(oy);
    }
    // inner-product accumulation: acc holds sum of v*k*2^-64 in [0, 2q); v canonical or forward-lazy (any 64-bit word)
    static HD T acc_zero() { return 0; }
    static HD void acc_mac(T& acc, T v, u64 key, const Mod& m) {
        u128w p = {0, 0};
        mac128(p, v, key);  // v < 2^64, key < q: v*key < q*2^64
        u64 r = redc_lazy(p, m.q, m.qneg);
        u64 s = acc + r;
        acc = s >= m.q2 ? s - m.q2 : s;
    }
    static HD T acc_fold(T acc, const Mod&) { return acc; }  // already kept in [0, 2q)
    static HD T acc_finish(T acc, const Mod& m) {  // remove the 2^-64: result in [0, 2q), valid as inverse-lazy
        return mul_shoup_lazy(acc, m.r1, m.r1_p, m.q);
    }
    static HD u64 acc_canon(T fin, const Mod& m) { return csub(fin, m.q); }
    // product of two canonical residues as an acc_mac operand carrying one more factor 2^-64 (in [0, 2q))
    static HD T premul(u64 a, u64 b, const Mod& m) {
        u128w p = {0, 0};
        mac128(p, a, b);
        return redc_lazy(p, m.q, m.qneg);
    }
    // finish of an accumulation whose operands came from premul: removes 2^-128
    static HD T acc_finish2(T acc, const Mod& m) {
        return mul_shoup_lazy(mul_shoup_lazy(acc, m.r1, m.r1_p, m.q), m.r1, m.r1_p, m.q);
    }
};

// ------------------------------------------------------------------------------- FpAr
// Conversions between residues and doubles through the bit pattern of 2^52 + x: for 0 <= x < 2^52 the
// double 2^52 + x has exponent 2^52 and x itself as its 52 mantissa bits (FpAr residues are below 2^50).
HD double u64_to_f64(u64 x) {  // exact for x < 2^52
    return __builtin_bit_cast(double, x | 0x4330000000000000ull) - 4503599627370496.0;
}
HD u64 f64_to_u64(double d) {  // exact for integer-valued 0 <= d < 2^52
    return __builtin_bit_cast(u64, d + 4503599627370496.0) & 0x000fffffffffffffull;
}

struct FpAr {
    typedef double T;
    static constexpr bool is_fp = true;
    struct Mod {
        double q, qinv;
    };
    struct Tw {
        double w;
    };
    static HD Mod mod(const PrimeConst& p) { return Mod{p.qd, p.qinv}; }
    // tables: tw_fp [prime][2][N] = fwd w, inv w (as doubles)
    static HD Tw tw(const u64*, const double* tf, u32 idx, u32 N, bool inverse) {
        return Tw{tf[(inverse ? (size_t)N : 0) + idx]};
    }
    static HD T mulmod_lazy(T a, T w, const Mod& m) {
        double h = a * w;
        double l = __builtin_fma(a, w, -h);
        double c = __builtin_rint(h * m.qinv);
        return __builtin_fma(-c, m.q, h) + l;
    }
    static HD T reduce(T x, const Mod& m) {  // |result| <= q/2 (+ rounding slack far below 1)
        double c = __builtin_rint(x * m.qinv);
        return __builtin_fma(-c, m.q, x);
    }
    // A word y < 2^61 given as ya + yl with ya = (y >> 30) * 2^30 (31 significant bits, an exact double) and
    // yl = y mod 2^30: an integer-valued double congruent to y modulo q with |result| <= (0.5 + 2^-19) q + 2^30.
    // The quotient ya / q is below 2^33 for q >= 2^28, so its estimate is off by less than 2^-19 before
    // rounding; ya - c*q is an integer below 2^50 in magnitude, hence the fma and the sum are exact.
    static HD T reduce_split(double ya, double yl, const Mod& m) {
        double c = __builtin_rint(ya * m.qinv);
        return __builtin_fma(-c, m.q, ya) + yl;
    }
    static HD T from_canon(u64 v, const Mod&) { return u64_to_f64(v); }
    static HD T from_raw(u64 v) { return __builtin_bit_cast(double, v); }
    static HD u64 to_raw(T v) { return __builtin_bit_cast(u64, v); }
    static HD T from_f64_lazy(double v, const Mod& m) { return reduce(v, m); }
    static HD T mul_canon(u64 a, u64 b, const PrimeConst&, const Mod& m) {
        return mulmod_lazy(u64_to_f64(a), u64_to_f64(b), m);  // |result| <= 0.875 q
    }
    template <bool RED>  // the reduction schedule of the integer arithmetic does not apply: ranges are restored per round
    static HD void bfly_fwd(T& X, T& Y, const Tw& t, const Mod& m) {
        double r = mulmod_lazy(Y, t.w, m);
        double x = X;
        X = x + r;
        Y = x - r;
    }
    static HD void bfly_inv(T& X, T& Y, const Tw& t, const Mod& m) {
        double s = X + Y, d = X - Y;
        X = s;
        Y = mulmod_lazy(d, t.w, m);
    }
    static HD T round_reduce(T v, const Mod& m) { return reduce(v, m); }
    static HD u64 canon(T v, const Mod& m) {
        double r = reduce(v, m);
        r = r < 0.0 ? r + m.q : r;
        return f64_to_u64(r);
    }
    static HD u64 canon_fwd(T v, const Mod& m) { return canon(v, m); }
    static HD u64 canon_inv(T v, const Mod& m) { return canon(v, m); }
    static HD double canon_f64(T v, const Mod& m) {
        double r = reduce(v, m);
        return r < 0.0 ? r + m.q : r;
    }
    // fmt: SRC_F64 stores the canonical value as a double's bit pattern, SRC_DIGITS as signed digits
    static HD void bfly_inv_last(T& X, T& Y, const InvScale& s, const Mod& m, u32 fmt, u64& ox, u64& oy) {
        double a = X + Y, d = X - Y;
        double rx = canon_f64(mulmod_lazy(a, s.sxd, m), m), ry = canon_f64(mulmod_lazy(d, s.syd, m), m);
        ox = fmt == SRC_F64 ? to_raw(rx) : f64_to_u64(rx);
        oy = fmt == SRC_F64 ? to_raw(ry) : f64_to_u64(ry);
        if (fmt == SRC_DIGITS) ox = digits_encode(ox), oy = digits_encode(oy);
    }
    static HD T acc_zero() { return 0.0; }
    static HD void acc_mac(T& acc, T v, u64 key, const Mod& m) { acc += mulmod_lazy(v, u64_to_f64(key), m); }
    static HD T acc_fold(T acc, const Mod& m) { return reduce(acc, m); }
    static HD T acc_finish(T acc, const Mod& m) { return reduce(acc, m); }
    static HD u64 acc_canon(T fin, const Mod& m) {
        double r = fin < 0.0 ? fin + m.q : fin;
        return f64_to_u64(r);
    }
    static HD T premul(u64 a, u64 b, const Mod& m) { return mulmod_lazy(u64_to_f64(a), u64_to_f64(b), m); }  // <= 0.875 q
    static HD T acc_finish2(T acc, const Mod& m) { return reduce(acc, m); }
};
