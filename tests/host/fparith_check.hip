// Host-side check of the FP64 modular arithmetic used by the HIP kernels (csrc/modarith.h).
// The functions are __host__ __device__; x86-64 FMA and CDNA4 FMA are both IEEE-754 binary64, so
// exactness shown here is exactness on the GPU.  Compares against 128-bit integer arithmetic:
//   * mulmod_lazy(a, w): congruent to a*w mod q, |r| <= (0.5 + 3A/8) q + 2^49 for |a| <= A q, A <= 8
//   * reduce / canon / conversions
//   * reduce_split: a 61-bit word brought below the modulus, and its product with a constant
//   * four forward and four inverse butterfly stages from the documented start ranges stay exact
// Prints "OK <count>" or the first failure.
#include <stdio.h>
#include <stdlib.h>
#include <math.h>
#include "../../paper_2310_16530_amd/csrc/modarith.h"

typedef __int128 i128;
static u64 rng_state = 0x9E3779B97F4A7C15ull;
static u64 rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return rng_state; }
static long long imod(i128 x, long long q) { long long r = (long long)(x % q); return r < 0 ? r + q : r; }

static int check_prime(u64 q, unsigned long long* count) {
    PrimeConst pc; pc.q = q; pc.qd = (double)q; pc.qinv = 1.0 / (double)q;
    const FpAr::Mod m = FpAr::mod(pc);
    const double A_list[] = {0.5, 1.0, 2.0, 4.0, 6.2, 8.0};
    for (double A : A_list) {
        const double lim = floor(A * (double)q);
        for (int it = 0; it < 200000; it++) {
            double a; u64 w;
            switch (it & 7) {
                case 0: a = lim; w = q - 1; break;
                case 1: a = -lim; w = q - 1; break;
                case 2: a = lim; w = 1; break;
                case 3: a = -lim; w = q / 2; break;
                case 4: a = lim - (double)(rnd() % 1000); w = q - 1 - rnd() % 1000; break;
                default: a = floor(((double)(rnd() >> 11) / 9007199254740992.0 * 2.0 - 1.0) * lim); w = rnd() % q; break;
            }
            const double r = FpAr::mulmod_lazy(a, (double)w, m);
            if (r != floor(r)) { printf("non-integer result q=%llu a=%.0f w=%llu\n", (unsigned long long)q, a, (unsigned long long)w); return 1; }
            const i128 exact = (i128)(long long)a * (i128)w;
            if (imod(exact, (long long)q) != imod((i128)(long long)r, (long long)q)) {
                printf("wrong residue q=%llu a=%.0f w=%llu r=%.0f\n", (unsigned long long)q, a, (unsigned long long)w, r); return 1; }
            const double bound = (0.5 + 3.0 * A / 8.0) * (double)q + 562949953421312.0;
            if (fabs(r) > bound) { printf("bound exceeded q=%llu A=%.1f a=%.0f w=%llu r=%.0f\n", (unsigned long long)q, A, a, (unsigned long long)w, r); return 1; }
            // reduce + canon
            const double red = FpAr::reduce(a, m);
            if (fabs(red) > 0.5 * (double)q + 1.0 || imod((i128)(long long)red, (long long)q) != imod((i128)(long long)a, (long long)q)) {
                printf("reduce failed q=%llu a=%.0f\n", (unsigned long long)q, a); return 1; }
            const u64 can = FpAr::canon(a, m);
            if (can >= q || (long long)can != imod((i128)(long long)a, (long long)q)) { printf("canon failed q=%llu a=%.0f\n", (unsigned long long)q, a); return 1; }
            (*count)++;
        }
    }
    // conversions
    for (int it = 0; it < 100000; it++) {
        const u64 x = it < 4 ? (it == 0 ? 0 : it == 1 ? q - 1 : it == 2 ? (1ull << 32) : (1ull << 32) - 1) : rnd() % q;
        if (f64_to_u64(u64_to_f64(x)) != x || (u64)u64_to_f64(x) != x) { printf("conversion failed %llu\n", (unsigned long long)x); return 1; }
        (*count)++;
    }
    // four forward stages from |x| <= q and four inverse stages from |x| <= q/2 on 16 values, worst-case signs
    for (int it = 0; it < 20000; it++) {
        double x[16]; long long ref[16]; double y[16]; long long refy[16];
        u64 w[15];
        for (int k = 0; k < 15; k++) w[k] = (it & 1) ? q - 1 - rnd() % 3 : rnd() % q;
        for (int k = 0; k < 16; k++) {
            const u64 v = (it & 2) ? q - 1 - rnd() % 3 : rnd() % q;
            x[k] = (double)v; ref[k] = (long long)v;
            const long long c = (it & 2) ? ((k & 1) ? (long long)(q / 2) : -(long long)(q / 2)) : (long long)(rnd() % q) - (long long)(q / 2);
            y[k] = (double)c; refy[k] = imod(c, (long long)q);
        }
        int ti = 0;
        for (int s = 0; s < 4; s++) {
            const int d = 8 >> s;
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                const FpAr::Tw tw = {(double)w[(1 << s) - 1 + (k >> (4 - s))]};
                FpAr::bfly_fwd<false>(x[k], x[k + d], tw, m);
                const long long t = imod((i128)ref[k + d] * (i128)(u64)tw.w, (long long)q);
                const long long X = ref[k];
                ref[k] = imod((i128)X + t, (long long)q); ref[k + d] = imod((i128)X - t, (long long)q);
                ti++;
            }
        }
        for (int s = 0; s < 4; s++) {
            const int d = 1 << s;
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                const FpAr::Tw tw = {(double)w[(k * 7 + s) % 15]};
                FpAr::bfly_inv(y[k], y[k + d], tw, m);
                const long long X = refy[k], Y = refy[k + d];
                refy[k] = imod((i128)X + Y, (long long)q);
                refy[k + d] = imod((i128)imod((i128)X - Y, (long long)q) * (i128)(u64)tw.w, (long long)q);
            }
        }
        for (int k = 0; k < 16; k++) {
            if (fabs(x[k]) >= 7.0 * (double)q || fabs(y[k]) > 8.0 * (double)q + 1.0 || fabs(y[k]) >= 9007199254740992.0) {
                printf("range exceeded q=%llu x=%.0f y=%.0f\n", (unsigned long long)q, x[k], y[k]); return 1; }
            if ((long long)FpAr::canon(x[k], m) != ref[k] || (long long)FpAr::canon(y[k], m) != refy[k]) {
                printf("stage mismatch q=%llu k=%d\n", (unsigned long long)q, k); return 1; }
        }
        (*count)++;
    }
    // a word below 2^61 brought below the modulus (ModDown sources) and then multiplied by a constant:
    // reduce_split needs q >= 2^28; eight such products (the most one accumulation round holds) stay exact
    if (q >= (1ull << 28)) {
        for (int it = 0; it < 200000; it++) {
            u64 y;
            switch (it & 7) {
                case 0: y = (1ull << 61) - 1; break;
                case 1: y = (1ull << 61) - (1ull << 30); break;
                case 2: y = (it >> 3) % 64 < 61 ? (1ull << ((it >> 3) % 61)) : 0; break;
                case 3: y = q * (rnd() % ((1ull << 61) / q)) + (q - 1) / 2 + (it & 8 ? 1 : 0); break;  // near half-way quotients
                default: y = rnd() >> 3; break;
            }
            const double ya = (double)(u32)(y >> 30) * 1073741824.0, yl = (double)(u32)(y & 0x3fffffffu);
            const double sred = FpAr::reduce_split(ya, yl, m);
            if (sred != floor(sred) || imod((i128)(long long)sred, (long long)q) != (long long)(y % q) ||
                fabs(sred) > (0.5 + 1.0 / 524288.0) * (double)q + 1073741824.0) {
                printf("reduce_split failed q=%llu y=%llu s=%.0f\n", (unsigned long long)q, (unsigned long long)y, sred); return 1; }
            const u64 w = (it & 16) ? q - 1 : rnd() % q;
            const double r = FpAr::mulmod_lazy(sred, (double)w, m);
            if (r != floor(r) || imod((i128)(long long)r, (long long)q) != imod((i128)(y % q) * (i128)w, (long long)q)) {
                printf("reduce_split product failed q=%llu y=%llu w=%llu\n", (unsigned long long)q, (unsigned long long)y, (unsigned long long)w); return 1; }
            if (8.0 * fabs(r) + 0.5 * (double)q >= 9007199254740992.0) {
                printf("eight reduce_split products do not fit q=%llu r=%.0f\n", (unsigned long long)q, r); return 1; }
            (*count)++;
        }
    }
    return 0;
}

int main(int argc, char** argv) {
    unsigned long long count = 0;
    for (int i = 1; i < argc; i++)
        if (check_prime(strtoull(argv[i], nullptr, 10), &count)) return 1;
    printf("OK %llu\n", count);
    return 0;
}
