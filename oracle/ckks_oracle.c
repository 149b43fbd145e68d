/*
 * CPU ORACLE for the RNS-CKKS key-switch path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow and meant to be checked by eye: every modular product is a
 * 128-bit multiply followed by `%`, the transform is the textbook iterative
 * butterfly network (pinned in the tests to the O(N^2) definition below), base
 * conversion is the uncorrected fast conversion written out term by term.  No
 * Barrett / Montgomery / Shoup / lazy reduction, no blocking or fusion.  It
 * shares no code, tables or constants with the HIP library; only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Object (paper, Section 2): a polynomial of Z_Q[X]/(X^N+1) is an L x N integer
 * matrix of 64-bit words, one row ("limb") per RNS prime; the major kernels are
 * the NTT and the base conversion.  The paper defines none of the steps itself
 * (it defers to the full-RNS CKKS scheme it cites), so each function states
 * the definition it evaluates.  Conventions: prime order q_0..q_{L-1},
 * p_0..p_{K-1}; residues canonical in [0, prime); ciphertext = (c0, c1) with
 * decryption c0 + c1*s; digit j = limbs j*alpha .. (j+1)*alpha-1, alpha = L/dnum
 * (the level functions and the key generator take alpha = ceil(L/dnum) and a shorter last digit
 * when dnum does not divide L; the full-level functions are written for digits of equal size).
 *
 * Parallelism: OpenMP over independent limbs only.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ threads */
/* Timing aid for the benchmark's CPU baseline: how many OpenMP threads the limb loops use, and a way to pin
 * that number (1 = single thread).  No effect on any result. */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
void orc_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif

/* ------------------------------------------------------------------ scalars */
uint64_t orc_mulmod(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)(((u128)a * b) % m); }
uint64_t orc_addmod(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)(((u128)a + b) % m); }
uint64_t orc_submod(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)(((u128)a + m - (b % m)) % m); }

uint64_t orc_powmod(uint64_t b, uint64_t e, uint64_t m) {
    uint64_t r = 1 % m;
    b %= m;
    while (e) {
        if (e & 1) r = orc_mulmod(r, b, m);
        b = orc_mulmod(b, b, m);
        e >>= 1;
    }
    return r;
}

/* m prime: a^(m-2) */
uint64_t orc_invmod(uint64_t a, uint64_t m) { return orc_powmod(a, m - 2, m); }

static uint32_t bitrev(uint32_t x, uint32_t bits) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

/* Numerically smallest psi in [2, m) with psi^N = -1 (mod m), N = 2^logN, m = 1 mod 2N.
 * All primitive 2N-th roots are the odd powers of any one of them; take their minimum. */
uint64_t orc_min_psi(uint64_t m, uint32_t logN) {
    uint64_t N = 1ull << logN;
    uint64_t root = 0;
    for (uint64_t x = 2; x < m; x++) {
        uint64_t y = orc_powmod(x, (m - 1) / (2 * N), m);
        if (orc_powmod(y, N, m) == m - 1) { root = y; break; }
    }
    uint64_t sq = orc_mulmod(root, root, m), cur = root, best = root;
    for (uint64_t k = 1; k < N; k++) {
        cur = orc_mulmod(cur, sq, m);
        if (cur < best) best = cur;
    }
    return best;
}

/* --------------------------------------------------------------- transforms */
/* Definition of the forward negacyclic NTT, one output:
 *   X^[j] = sum_t x_t * psi^(t*(2*brev(j)+1))  (mod m)
 * i.e. the polynomial evaluated at the odd power psi^(2*brev(j)+1); outputs are
 * in bit-reversed order of the evaluation points. */
uint64_t orc_ntt_def_at(const uint64_t* x, uint32_t logN, uint64_t m, uint64_t psi, uint32_t j) {
    uint64_t N = 1ull << logN;
    uint64_t point = orc_powmod(psi, 2ull * bitrev(j, logN) + 1, m);
    uint64_t acc = 0, pw = 1;
    for (uint64_t t = 0; t < N; t++) {
        acc = orc_addmod(acc, orc_mulmod(x[t], pw, m), m);
        pw = orc_mulmod(pw, point, m);
    }
    return acc;
}

void orc_ntt_def(const uint64_t* x, uint64_t* out, uint32_t logN, uint64_t m, uint64_t psi) {
    uint32_t N = 1u << logN;
    for (uint32_t j = 0; j < N; j++) out[j] = orc_ntt_def_at(x, logN, m, psi, j);
}

/* Textbook in-place decimation network computing the same map in O(N log N):
 * stage with `groups` groups of half-width t; group i uses psi^brev(groups+i). */
void orc_ntt(uint64_t* x, uint32_t logN, uint64_t m, uint64_t psi) {
    uint32_t N = 1u << logN;
    uint64_t* w = (uint64_t*)malloc(sizeof(uint64_t) * N);
    for (uint32_t k = 0; k < N; k++) w[k] = orc_powmod(psi, bitrev(k, logN), m);
    uint32_t t = N;
    for (uint32_t groups = 1; groups < N; groups *= 2) {
        t /= 2;
        for (uint32_t i = 0; i < groups; i++) {
            uint64_t s = w[groups + i];
            for (uint32_t j = 2 * i * t; j < 2 * i * t + t; j++) {
                uint64_t u = x[j];
                uint64_t v = orc_mulmod(x[j + t], s, m);
                x[j] = orc_addmod(u, v, m);
                x[j + t] = orc_submod(u, v, m);
            }
        }
    }
    free(w);
}

/* Inverse of orc_ntt: the same network run backwards with inverse twiddles,
 * then the factor N^-1.  Natural-order coefficients out. */
void orc_intt(uint64_t* x, uint32_t logN, uint64_t m, uint64_t psi) {
    uint32_t N = 1u << logN;
    uint64_t psi_inv = orc_invmod(psi, m);
    uint64_t* w = (uint64_t*)malloc(sizeof(uint64_t) * N);
    for (uint32_t k = 0; k < N; k++) w[k] = orc_powmod(psi_inv, bitrev(k, logN), m);
    uint32_t t = 1;
    for (uint32_t groups = N / 2; groups >= 1; groups /= 2) {
        for (uint32_t i = 0; i < groups; i++) {
            uint64_t s = w[groups + i];
            for (uint32_t j = 2 * i * t; j < 2 * i * t + t; j++) {
                uint64_t u = x[j], v = x[j + t];
                x[j] = orc_addmod(u, v, m);
                x[j + t] = orc_mulmod(orc_submod(u, v, m), s, m);
            }
        }
        t *= 2;
    }
    uint64_t n_inv = orc_invmod(N % m, m);
    for (uint32_t j = 0; j < N; j++) x[j] = orc_mulmod(x[j], n_inv, m);
    free(w);
}

/* x: [batch][n_limbs][N]; limb l uses primes[l], psi[l]. */
void orc_ntt_batch(uint64_t* x, uint32_t logN, uint32_t n_limbs, uint32_t batch,
                   const uint64_t* primes, const uint64_t* psi, int inverse) {
    size_t N = (size_t)1 << logN;
    long total = (long)n_limbs * batch;
#pragma omp parallel for schedule(dynamic)
    for (long id = 0; id < total; id++) {
        uint32_t l = (uint32_t)(id % n_limbs);
        if (inverse) orc_intt(x + (size_t)id * N, logN, primes[l], psi[l]);
        else orc_ntt(x + (size_t)id * N, logN, primes[l], psi[l]);
    }
}

/* ---------------------------------------------------------- base conversion */
/* Fast base conversion from the basis {src[0..ns)} to one target prime b:
 *   y_i   = x_i * [(S/src_i)^-1]_{src_i}  mod src_i          (canonical)
 *   out   = sum_i y_i * ((S/src_i) mod b)  mod b,   S = prod src
 * with no correction of the overflow u*S (0 <= u < ns).
 * x: ns rows of N words (row stride `stride`), out: N words. */
void orc_conv(const uint64_t* x, size_t stride, size_t N, const uint64_t* src, uint32_t ns,
              uint64_t b, uint64_t* out) {
    uint64_t* hat_inv = (uint64_t*)malloc(sizeof(uint64_t) * ns);
    uint64_t* hat_b = (uint64_t*)malloc(sizeof(uint64_t) * ns);
    for (uint32_t i = 0; i < ns; i++) {
        uint64_t hi = 1, hb = 1;
        for (uint32_t k = 0; k < ns; k++) {
            if (k == i) continue;
            hi = orc_mulmod(hi, src[k] % src[i], src[i]);
            hb = orc_mulmod(hb, src[k] % b, b);
        }
        hat_inv[i] = orc_invmod(hi, src[i]);
        hat_b[i] = hb;
    }
    for (size_t n = 0; n < N; n++) {
        uint64_t acc = 0;
        for (uint32_t i = 0; i < ns; i++) {
            uint64_t y = orc_mulmod(x[i * stride + n], hat_inv[i], src[i]);
            acc = orc_addmod(acc, orc_mulmod(y, hat_b[i], b), b);
        }
        out[n] = acc;
    }
    free(hat_inv);
    free(hat_b);
}

/* ModUp (digit decomposition + extension), coefficient form.
 * in: [L][N]; out: [dnum][L+K][N].  Digit j keeps its own alpha limbs and every
 * other limb of the extended basis is the fast conversion of those alpha limbs. */
void orc_modup(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t L, uint32_t K,
               uint32_t dnum, const uint64_t* primes) {
    size_t N = (size_t)1 << logN;
    uint32_t alpha = L / dnum, D = L + K;
    long total = (long)dnum * D;
#pragma omp parallel for schedule(dynamic)
    for (long id = 0; id < total; id++) {
        uint32_t j = (uint32_t)(id / D), t = (uint32_t)(id % D);
        uint64_t* dst = out + ((size_t)j * D + t) * N;
        if (t >= j * alpha && t < (j + 1) * alpha) {
            memcpy(dst, in + (size_t)t * N, N * sizeof(uint64_t));
        } else {
            orc_conv(in + (size_t)j * alpha * N, N, N, primes + j * alpha, alpha, primes[t], dst);
        }
    }
}

/* ModDown, coefficient form.  in: [L+K][N]; out: [L][N]:
 *   out_i = (in_i - Conv_{P -> q_i}(in restricted to the special limbs)) * [P^-1]_{q_i}  mod q_i
 * (floor-type: no rounding term is added). */
void orc_moddown(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t L, uint32_t K,
                 const uint64_t* primes) {
    size_t N = (size_t)1 << logN;
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)L; i++) {
        uint64_t q = primes[i];
        uint64_t* conv = (uint64_t*)malloc(sizeof(uint64_t) * N);
        orc_conv(in + (size_t)L * N, N, N, primes + L, K, q, conv);
        uint64_t P = 1;
        for (uint32_t k = 0; k < K; k++) P = orc_mulmod(P, primes[L + k] % q, q);
        uint64_t Pinv = orc_invmod(P, q);
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_mulmod(orc_submod(in[(size_t)i * N + n], conv[n], q), Pinv, q);
        free(conv);
    }
}

/* ------------------------------------------------------------- automorphism */
/* sigma_g : X -> X^g on coefficients.  X^t -> X^(t*g mod 2N), with X^N = -1. */
void orc_automorph_coeff(const uint64_t* in, uint64_t* out, uint32_t logN, uint64_t m, uint32_t g) {
    uint64_t N = 1ull << logN;
    for (uint64_t t = 0; t < N; t++) {
        uint64_t u = (t * g) % (2 * N);
        if (u < N) out[u] = in[t];
        else out[u - N] = (m - in[t]) % m;
    }
}

/* The same map on evaluation form: slot j holds the value at psi^(2*brev(j)+1);
 * sigma_g(f)(z) = f(z^g), so out[j] = in[j'] with 2*brev(j')+1 = g*(2*brev(j)+1) mod 2N. */
void orc_automorph_eval(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t g) {
    uint64_t N = 1ull << logN;
    for (uint32_t j = 0; j < N; j++) {
        uint64_t e = ((uint64_t)g * (2ull * bitrev(j, logN) + 1)) % (2 * N);
        uint32_t jp = bitrev((uint32_t)((e - 1) / 2), logN);
        out[j] = in[jp];
    }
}

/* ------------------------------------------------------------- compositions */
typedef struct {
    uint32_t logN, L, K, dnum;
    const uint64_t* primes; /* L+K */
    const uint64_t* psi;    /* L+K */
} orc_params;

static void limbs_ntt(uint64_t* x, const orc_params* p, uint32_t first, uint32_t count, uint32_t groups,
                      uint32_t group_stride_limbs, int inverse) {
    size_t N = (size_t)1 << p->logN;
    long total = (long)count * groups;
#pragma omp parallel for schedule(dynamic)
    for (long id = 0; id < total; id++) {
        uint32_t gidx = (uint32_t)(id / count), l = first + (uint32_t)(id % count);
        uint64_t* row = x + ((size_t)gidx * group_stride_limbs + l) * N;
        if (inverse) orc_intt(row, p->logN, p->primes[l], p->psi[l]);
        else orc_ntt(row, p->logN, p->primes[l], p->psi[l]);
    }
}

/* Inner product of the extended digits with a switching key, evaluation form:
 *   c'_t[i] = sum_j dhat_j[i] * key[j][t][i]  mod prime_i,  t in {0,1}, i over L+K limbs.
 * If galois != 1 the digits are first permuted by the evaluation-form automorphism. */
static void key_inner_product(const uint64_t* dhat /*[dnum][D][N]*/, const uint64_t* key /*[dnum][2][D][N]*/,
                              uint64_t* cp /*[2][D][N]*/, const orc_params* p, uint32_t galois) {
    size_t N = (size_t)1 << p->logN;
    uint32_t D = p->L + p->K;
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)D; i++) {
        uint64_t m = p->primes[i];
        uint64_t* perm = (uint64_t*)malloc(sizeof(uint64_t) * N);
        for (uint32_t t = 0; t < 2; t++) memset(cp + ((size_t)t * D + i) * N, 0, N * sizeof(uint64_t));
        for (uint32_t j = 0; j < p->dnum; j++) {
            const uint64_t* src = dhat + ((size_t)j * D + i) * N;
            if (galois != 1) { orc_automorph_eval(src, perm, p->logN, galois); src = perm; }
            for (uint32_t t = 0; t < 2; t++) {
                const uint64_t* k = key + (((size_t)j * 2 + t) * D + i) * N;
                uint64_t* dst = cp + ((size_t)t * D + i) * N;
                for (size_t n = 0; n < N; n++)
                    dst[n] = orc_addmod(dst[n], orc_mulmod(src[n], k[n], m), m);
            }
        }
        free(perm);
    }
}

/* cp: [2][D][N] evaluation form -> ks: [2][L][N] evaluation form:
 * ks_t = NTT(ModDown(INTT(c'_t))). cp is overwritten. */
static void moddown_eval(uint64_t* cp, uint64_t* ks, const orc_params* p) {
    size_t N = (size_t)1 << p->logN;
    uint32_t D = p->L + p->K;
    limbs_ntt(cp, p, 0, D, 2, D, 1);
    for (uint32_t t = 0; t < 2; t++)
        orc_moddown(cp + (size_t)t * D * N, ks + (size_t)t * p->L * N, p->logN, p->L, p->K, p->primes);
    limbs_ntt(ks, p, 0, p->L, 2, p->L, 0);
}

/* dhat = NTT(ModUp(INTT(d))) on all L+K limbs of every digit. d: [L][N] eval; dhat: [dnum][D][N]. */
static void decompose_extend(const uint64_t* d, uint64_t* dhat, const orc_params* p) {
    size_t N = (size_t)1 << p->logN;
    uint32_t D = p->L + p->K;
    uint64_t* x = (uint64_t*)malloc(sizeof(uint64_t) * p->L * N);
    memcpy(x, d, sizeof(uint64_t) * p->L * N);
    limbs_ntt(x, p, 0, p->L, 1, p->L, 1);
    orc_modup(x, dhat, p->logN, p->L, p->K, p->dnum, p->primes);
    limbs_ntt(dhat, p, 0, D, p->dnum, D, 0);
    free(x);
}

/* Hybrid key switch: d [L][N] eval, key [dnum][2][L+K][N] eval -> out [2][L][N] eval. */
void orc_keyswitch(const uint64_t* d, const uint64_t* key, uint64_t* out, uint32_t logN, uint32_t L,
                   uint32_t K, uint32_t dnum, const uint64_t* primes, const uint64_t* psi) {
    orc_params p = {logN, L, K, dnum, primes, psi};
    size_t N = (size_t)1 << logN;
    uint32_t D = L + K;
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    decompose_extend(d, dhat, &p);
    key_inner_product(dhat, key, cp, &p, 1);
    moddown_eval(cp, out, &p);
    free(dhat);
    free(cp);
}

/* Homomorphic multiply with relinearisation (no rescale).  ct = [2][L][N] eval, index 0 = c0.
 *   d0 = b1*b2, d1 = a1*b2 + a2*b1, d2 = a1*a2;  out = (d0 + ks0, d1 + ks1), ks = KeySwitch(d2, evk). */
void orc_hmult_relin(const uint64_t* ct1, const uint64_t* ct2, const uint64_t* evk, uint64_t* out,
                     uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes,
                     const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint64_t* d2 = (uint64_t*)malloc(sizeof(uint64_t) * L * N);
    uint64_t* ks = (uint64_t*)malloc(sizeof(uint64_t) * 2 * L * N);
    for (uint32_t i = 0; i < L; i++) {
        uint64_t m = primes[i];
        const uint64_t *a1 = ct1 + ((size_t)L + i) * N, *a2 = ct2 + ((size_t)L + i) * N;
        for (size_t n = 0; n < N; n++) d2[(size_t)i * N + n] = orc_mulmod(a1[n], a2[n], m);
    }
    orc_keyswitch(d2, evk, ks, logN, L, K, dnum, primes, psi);
    for (uint32_t i = 0; i < L; i++) {
        uint64_t m = primes[i];
        const uint64_t *b1 = ct1 + (size_t)i * N, *a1 = ct1 + ((size_t)L + i) * N;
        const uint64_t *b2 = ct2 + (size_t)i * N, *a2 = ct2 + ((size_t)L + i) * N;
        for (size_t n = 0; n < N; n++) {
            uint64_t d0 = orc_mulmod(b1[n], b2[n], m);
            uint64_t d1 = orc_addmod(orc_mulmod(a1[n], b2[n], m), orc_mulmod(a2[n], b1[n], m), m);
            out[(size_t)i * N + n] = orc_addmod(d0, ks[(size_t)i * N + n], m);
            out[((size_t)L + i) * N + n] = orc_addmod(d1, ks[((size_t)L + i) * N + n], m);
        }
    }
    free(d2);
    free(ks);
}

/* Homomorphic rotation by Galois element g: out = (sigma_g(b) + ks0, ks1), ks = KeySwitch(sigma_g(a), rk_g). */
void orc_hrot(const uint64_t* ct, uint32_t g, const uint64_t* rk, uint64_t* out, uint32_t logN,
              uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes, const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint64_t* rot = (uint64_t*)malloc(sizeof(uint64_t) * 2 * L * N);
    for (uint32_t i = 0; i < 2 * L; i++) orc_automorph_eval(ct + (size_t)i * N, rot + (size_t)i * N, logN, g);
    orc_keyswitch(rot + (size_t)L * N, rk, out, logN, L, K, dnum, primes, psi);
    for (uint32_t i = 0; i < L; i++)
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], rot[(size_t)i * N + n], primes[i]);
    free(rot);
}

/* Hoisted rotate-multiply-accumulate.  The decomposition of a is done once; for
 * every rotation r the evaluation-form automorphism is applied to the extended
 * digits, then inner product with rk_r, ModDown, add sigma(b), and
 *   out += pt_r * (sigma_r(b) + ks0, ks1)        (both components).
 * If per_rot != NULL it receives the un-multiplied rotated ciphertexts [n_rot][2][L][N]. */
void orc_hrot_hoisted_mac(const uint64_t* ct, uint32_t n_rot, const uint32_t* galois,
                          const uint64_t* const* rk, const uint64_t* pt /*[n_rot][L][N]*/, uint64_t* out,
                          uint64_t* per_rot, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                          const uint64_t* primes, const uint64_t* psi) {
    orc_params p = {logN, L, K, dnum, primes, psi};
    size_t N = (size_t)1 << logN;
    uint32_t D = L + K;
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    uint64_t* ks = (uint64_t*)malloc(sizeof(uint64_t) * 2 * L * N);
    uint64_t* sb = (uint64_t*)malloc(sizeof(uint64_t) * N);
    decompose_extend(ct + (size_t)L * N, dhat, &p);
    memset(out, 0, sizeof(uint64_t) * 2 * L * N);
    for (uint32_t r = 0; r < n_rot; r++) {
        key_inner_product(dhat, rk[r], cp, &p, galois[r]);
        moddown_eval(cp, ks, &p);
        for (uint32_t i = 0; i < L; i++) {
            uint64_t m = primes[i];
            orc_automorph_eval(ct + (size_t)i * N, sb, logN, galois[r]);
            const uint64_t* ptr = pt + ((size_t)r * L + i) * N;
            for (size_t n = 0; n < N; n++) {
                uint64_t r0 = orc_addmod(sb[n], ks[(size_t)i * N + n], m);
                uint64_t r1 = ks[((size_t)L + i) * N + n];
                if (per_rot) {
                    per_rot[(((size_t)r * 2) * L + i) * N + n] = r0;
                    per_rot[(((size_t)r * 2 + 1) * L + i) * N + n] = r1;
                }
                out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], orc_mulmod(ptr[n], r0, m), m);
                out[((size_t)L + i) * N + n] =
                    orc_addmod(out[((size_t)L + i) * N + n], orc_mulmod(ptr[n], r1, m), m);
            }
        }
    }
    free(dhat);
    free(cp);
    free(ks);
    free(sb);
}

/* ------------------------------------------------- levels below L and rescale */
/* A ciphertext at level ell (1 <= ell <= L) lives on the limbs q_0..q_{ell-1}: [2][ell][N].
 * The paper's CNN consumes one level per multiplication (Section 4: each layer's "multiplicative
 * level consumption"), i.e. every HMult is followed by a rescale and later operations run on
 * fewer limbs.  Definitions evaluated here:
 *
 * Rescale (floor type, like ModDown): with X the value in [0, Q_ell) of a coefficient and
 * q = q_{ell-1}, the result is (X - [X]_q) / q modulo Q_{ell-1}, limb by limb
 *     out_i = (in_i - NTT_i([INTT(in_{ell-1})] mod q_i)) * [q^-1]_{q_i}  mod q_i,   i < ell-1,
 * [.] the canonical representative in [0, q).
 *
 * Key switch at level ell with the full-level key: the extended basis is q_0..q_{ell-1},
 * p_0..p_{K-1}; digit j holds the active limbs j*alpha .. min((j+1)*alpha, ell)-1 (the last digit
 * may be partial, and its conversion constants are those of the limbs it really has); there are
 * beta = ceil(ell/alpha) digits; the key is read on the active limbs and the special limbs of
 * its first beta digits.  (The gadget of digit j is P on the digit's own limbs and 0 elsewhere,
 * which stays the CRT idempotent of the digit's active part modulo Q_ell, so the same key works.) */

void orc_rescale(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t ell, const uint64_t* primes,
                 const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint64_t qlast = primes[ell - 1];
    uint64_t* x = (uint64_t*)malloc(sizeof(uint64_t) * N);
    memcpy(x, in + (size_t)(ell - 1) * N, sizeof(uint64_t) * N);
    orc_intt(x, logN, qlast, psi[ell - 1]);
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)ell - 1; i++) {
        uint64_t q = primes[i];
        uint64_t qinv = orc_invmod(qlast % q, q);
        uint64_t* r = (uint64_t*)malloc(sizeof(uint64_t) * N);
        for (size_t n = 0; n < N; n++) r[n] = x[n] % q;
        orc_ntt(r, logN, q, psi[i]);
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_mulmod(orc_submod(in[(size_t)i * N + n], r[n], q), qinv, q);
        free(r);
    }
    free(x);
}

/* ModUp with digits of alpha limbs over ell active limbs (last digit possibly partial).
 * in: [ell][N] coefficient form; vprimes: the ell + K primes of the extended basis in order;
 * out: [beta][ell+K][N]. */
void orc_modup_level(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t ell, uint32_t K, uint32_t alpha,
                     const uint64_t* vprimes) {
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K, beta = (ell + alpha - 1) / alpha;
    long total = (long)beta * D;
#pragma omp parallel for schedule(dynamic)
    for (long id = 0; id < total; id++) {
        uint32_t j = (uint32_t)(id / D), t = (uint32_t)(id % D);
        uint32_t lo = j * alpha, hi = (j + 1) * alpha < ell ? (j + 1) * alpha : ell;
        uint64_t* dst = out + ((size_t)j * D + t) * N;
        if (t >= lo && t < hi) memcpy(dst, in + (size_t)t * N, N * sizeof(uint64_t));
        else orc_conv(in + (size_t)lo * N, N, N, vprimes + lo, hi - lo, vprimes[t], dst);
    }
}

/* Everything a level-ell operation needs: the primes/roots of the extended basis at that level and
 * the key restricted to it ([beta][2][ell+K][N], gathered from [dnum][2][L+K][N]). */
typedef struct {
    orc_params p; /* L = ell, dnum = beta, primes/psi = the arrays below */
    uint32_t alpha;
    uint64_t *vprimes, *vpsi;
} orc_level;

static void level_open(orc_level* v, uint32_t ell, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                       const uint64_t* primes, const uint64_t* psi) {
    uint32_t D = ell + K;
    v->alpha = (L + dnum - 1) / dnum; /* digits of ceil(L/dnum) limbs; the last one is shorter when dnum does not divide L */
    v->vprimes = (uint64_t*)malloc(sizeof(uint64_t) * D);
    v->vpsi = (uint64_t*)malloc(sizeof(uint64_t) * D);
    for (uint32_t i = 0; i < D; i++) {
        uint32_t src = i < ell ? i : L + (i - ell);
        v->vprimes[i] = primes[src];
        v->vpsi[i] = psi[src];
    }
    orc_params p = {logN, ell, K, (ell + v->alpha - 1) / v->alpha, v->vprimes, v->vpsi};
    v->p = p;
}

static void level_close(orc_level* v) {
    free(v->vprimes);
    free(v->vpsi);
}

static uint64_t* level_key(const orc_level* v, const uint64_t* key, uint32_t L) {
    size_t N = (size_t)1 << v->p.logN;
    uint32_t ell = v->p.L, K = v->p.K, D = ell + K, Dfull = L + K;
    uint64_t* kc = (uint64_t*)malloc(sizeof(uint64_t) * v->p.dnum * 2 * D * N);
    for (uint32_t j = 0; j < v->p.dnum; j++)
        for (uint32_t t = 0; t < 2; t++)
            for (uint32_t i = 0; i < D; i++) {
                uint32_t src = i < ell ? i : L + (i - ell);
                memcpy(kc + (((size_t)j * 2 + t) * D + i) * N, key + (((size_t)j * 2 + t) * Dfull + src) * N,
                       sizeof(uint64_t) * N);
            }
    return kc;
}

/* dhat = NTT(ModUp(INTT(d))) at a level: d [ell][N] eval -> dhat [beta][ell+K][N] eval. */
static void decompose_extend_level(const uint64_t* d, uint64_t* dhat, const orc_level* v) {
    const orc_params* p = &v->p;
    size_t N = (size_t)1 << p->logN;
    uint32_t D = p->L + p->K;
    uint64_t* x = (uint64_t*)malloc(sizeof(uint64_t) * p->L * N);
    memcpy(x, d, sizeof(uint64_t) * p->L * N);
    limbs_ntt(x, p, 0, p->L, 1, p->L, 1);
    orc_modup_level(x, dhat, p->logN, p->L, p->K, v->alpha, p->primes);
    limbs_ntt(dhat, p, 0, D, p->dnum, D, 0);
    free(x);
}

/* d [ell][N] eval, key [dnum][2][L+K][N] eval (full level) -> out [2][ell][N] eval. */
void orc_keyswitch_level(const uint64_t* d, const uint64_t* key, uint64_t* out, uint32_t ell, uint32_t logN,
                         uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes, const uint64_t* psi) {
    orc_level v;
    level_open(&v, ell, logN, L, K, dnum, primes, psi);
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K;
    uint64_t* kc = level_key(&v, key, L);
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * v.p.dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    decompose_extend_level(d, dhat, &v);
    key_inner_product(dhat, kc, cp, &v.p, 1);
    moddown_eval(cp, out, &v.p);
    free(dhat);
    free(cp);
    free(kc);
    level_close(&v);
}

/* HMult + relinearisation of two level-ell ciphertexts [2][ell][N] (no rescale). */
void orc_hmult_relin_level(const uint64_t* ct1, const uint64_t* ct2, const uint64_t* evk, uint64_t* out,
                           uint32_t ell, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                           const uint64_t* primes, const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint64_t* d2 = (uint64_t*)malloc(sizeof(uint64_t) * ell * N);
    uint64_t* ks = (uint64_t*)malloc(sizeof(uint64_t) * 2 * ell * N);
    for (uint32_t i = 0; i < ell; i++) {
        const uint64_t *a1 = ct1 + ((size_t)ell + i) * N, *a2 = ct2 + ((size_t)ell + i) * N;
        for (size_t n = 0; n < N; n++) d2[(size_t)i * N + n] = orc_mulmod(a1[n], a2[n], primes[i]);
    }
    orc_keyswitch_level(d2, evk, ks, ell, logN, L, K, dnum, primes, psi);
    for (uint32_t i = 0; i < ell; i++) {
        uint64_t m = primes[i];
        const uint64_t *b1 = ct1 + (size_t)i * N, *a1 = ct1 + ((size_t)ell + i) * N;
        const uint64_t *b2 = ct2 + (size_t)i * N, *a2 = ct2 + ((size_t)ell + i) * N;
        for (size_t n = 0; n < N; n++) {
            uint64_t d0 = orc_mulmod(b1[n], b2[n], m);
            uint64_t d1 = orc_addmod(orc_mulmod(a1[n], b2[n], m), orc_mulmod(a2[n], b1[n], m), m);
            out[(size_t)i * N + n] = orc_addmod(d0, ks[(size_t)i * N + n], m);
            out[((size_t)ell + i) * N + n] = orc_addmod(d1, ks[((size_t)ell + i) * N + n], m);
        }
    }
    free(d2);
    free(ks);
}

/* Rotation of a level-ell ciphertext: (sigma_g(b) + ks0, ks1), ks = KeySwitch_ell(sigma_g(a), rk_g). */
void orc_hrot_level(const uint64_t* ct, uint32_t g, const uint64_t* rk, uint64_t* out, uint32_t ell,
                    uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes,
                    const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint64_t* rot = (uint64_t*)malloc(sizeof(uint64_t) * 2 * ell * N);
    for (uint32_t i = 0; i < 2 * ell; i++) orc_automorph_eval(ct + (size_t)i * N, rot + (size_t)i * N, logN, g);
    orc_keyswitch_level(rot + (size_t)ell * N, rk, out, ell, logN, L, K, dnum, primes, psi);
    for (uint32_t i = 0; i < ell; i++)
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], rot[(size_t)i * N + n], primes[i]);
    free(rot);
}

/* Hoisted rotate-multiply-accumulate at level ell: as orc_hrot_hoisted_mac on the level's basis.
 * ct [2][ell][N], pt [n_rot][ell][N], out [2][ell][N]; keys are full-level. */
void orc_hrot_hoisted_mac_level(const uint64_t* ct, uint32_t n_rot, const uint32_t* galois,
                                const uint64_t* const* rk, const uint64_t* pt, uint64_t* out, uint32_t ell,
                                uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes,
                                const uint64_t* psi) {
    orc_level v;
    level_open(&v, ell, logN, L, K, dnum, primes, psi);
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K;
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * v.p.dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    uint64_t* ks = (uint64_t*)malloc(sizeof(uint64_t) * 2 * ell * N);
    uint64_t* sb = (uint64_t*)malloc(sizeof(uint64_t) * N);
    decompose_extend_level(ct + (size_t)ell * N, dhat, &v);
    memset(out, 0, sizeof(uint64_t) * 2 * ell * N);
    for (uint32_t r = 0; r < n_rot; r++) {
        uint64_t* kc = level_key(&v, rk[r], L);
        key_inner_product(dhat, kc, cp, &v.p, galois[r]);
        moddown_eval(cp, ks, &v.p);
        free(kc);
        for (uint32_t i = 0; i < ell; i++) {
            uint64_t m = primes[i];
            orc_automorph_eval(ct + (size_t)i * N, sb, logN, galois[r]);
            const uint64_t* ptr = pt + ((size_t)r * ell + i) * N;
            for (size_t n = 0; n < N; n++) {
                uint64_t r0 = orc_addmod(sb[n], ks[(size_t)i * N + n], m);
                uint64_t r1 = ks[((size_t)ell + i) * N + n];
                out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], orc_mulmod(ptr[n], r0, m), m);
                out[((size_t)ell + i) * N + n] =
                    orc_addmod(out[((size_t)ell + i) * N + n], orc_mulmod(ptr[n], r1, m), m);
            }
        }
    }
    free(dhat);
    free(cp);
    free(ks);
    free(sb);
    level_close(&v);
}

/* Double-hoisted rotate-multiply-accumulate (the linear-transform evaluation of the bootstrapping
 * work the paper builds on): besides sharing the decomposition, the plaintext products are summed in
 * the extended basis and ONE ModDown is applied to the sum,
 *     C_t[i]  = sum_r pt_r[i] * c'_{r,t}[i]        on all ell+K limbs,  c'_r as in the hoisted version,
 *     out_t   = NTT(ModDown(INTT(C_t))) + (t == 0 ? sum_r pt_r * sigma_{g_r}(b) : 0).
 * pt: [n_rot][ell+K][N], the plaintext polynomial reduced modulo every prime of the level's extended
 * basis (q_0..q_{ell-1}, p_0..p_{K-1}), evaluation form.  The result differs from the singly hoisted
 * one bit for bit (ModDown of a sum is not the sum of ModDowns) and carries less rounding noise. */
void orc_hrot_dh_mac_level(const uint64_t* ct, uint32_t n_rot, const uint32_t* galois, const uint64_t* const* rk,
                           const uint64_t* pt, uint64_t* out, uint32_t ell, uint32_t logN, uint32_t L, uint32_t K,
                           uint32_t dnum, const uint64_t* primes, const uint64_t* psi) {
    orc_level v;
    level_open(&v, ell, logN, L, K, dnum, primes, psi);
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K;
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * v.p.dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    uint64_t* C = (uint64_t*)calloc(2 * D * N, sizeof(uint64_t));
    uint64_t* sb = (uint64_t*)malloc(sizeof(uint64_t) * N);
    decompose_extend_level(ct + (size_t)ell * N, dhat, &v);
    memset(out, 0, sizeof(uint64_t) * 2 * ell * N);
    for (uint32_t r = 0; r < n_rot; r++) {
        uint64_t* kc = level_key(&v, rk[r], L);
        key_inner_product(dhat, kc, cp, &v.p, galois[r]);
        free(kc);
        for (uint32_t t = 0; t < 2; t++)
            for (uint32_t i = 0; i < D; i++) {
                uint64_t m = v.vprimes[i];
                const uint64_t* ptr = pt + ((size_t)r * D + i) * N;
                const uint64_t* src = cp + ((size_t)t * D + i) * N;
                uint64_t* dst = C + ((size_t)t * D + i) * N;
                for (size_t n = 0; n < N; n++) dst[n] = orc_addmod(dst[n], orc_mulmod(ptr[n], src[n], m), m);
            }
        for (uint32_t i = 0; i < ell; i++) { /* the b part never leaves the q-limbs */
            uint64_t m = primes[i];
            orc_automorph_eval(ct + (size_t)i * N, sb, logN, galois[r]);
            const uint64_t* ptr = pt + ((size_t)r * D + i) * N;
            for (size_t n = 0; n < N; n++)
                out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], orc_mulmod(ptr[n], sb[n], m), m);
        }
    }
    uint64_t* ks = (uint64_t*)malloc(sizeof(uint64_t) * 2 * ell * N);
    moddown_eval(C, ks, &v.p);
    for (uint32_t i = 0; i < 2 * ell; i++) {
        uint64_t m = primes[i % ell];
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_addmod(out[(size_t)i * N + n], ks[(size_t)i * N + n], m);
    }
    free(ks);
    free(dhat);
    free(cp);
    free(C);
    free(sb);
    level_close(&v);
}

/* ------------------------------------------- ModDown merged with the rescale that follows it */
/* Division by P * q_last in ONE floor-type step: the last active limb is treated as one more special
 * limb.  in: [ell+K][N] coefficient form on the level's extended basis vprimes = q_0..q_{ell-1},
 * p_0..p_{K-1}; S = {q_{ell-1}, p_0, .., p_{K-1}} = vprimes[ell-1 ..], PS its product;  out: [ell-1][N]:
 *   out_i = (in_i - Conv_{S -> q_i}(in restricted to S)) * [PS^-1]_{q_i}  mod q_i,   i < ell-1,
 * Conv the same uncorrected fast base conversion as everywhere else.  As an integer the result is
 * floor(X / PS) - u with 0 <= u <= K.  Not bit-identical to ModDown followed by rescale (two floors with
 * two overshoots), but never further than K+1 from it. */
void orc_moddown_merged(const uint64_t* in, uint64_t* out, uint32_t logN, uint32_t ell, uint32_t K,
                        const uint64_t* vprimes) {
    size_t N = (size_t)1 << logN;
    uint32_t T = ell - 1, ns = K + 1;
#pragma omp parallel for schedule(dynamic)
    for (long i = 0; i < (long)T; i++) {
        uint64_t q = vprimes[i];
        uint64_t* conv = (uint64_t*)malloc(sizeof(uint64_t) * N);
        orc_conv(in + (size_t)T * N, N, N, vprimes + T, ns, q, conv);
        uint64_t PS = 1;
        for (uint32_t k = 0; k < ns; k++) PS = orc_mulmod(PS, vprimes[T + k] % q, q);
        uint64_t PSinv = orc_invmod(PS, q);
        for (size_t n = 0; n < N; n++)
            out[(size_t)i * N + n] = orc_mulmod(orc_submod(in[(size_t)i * N + n], conv[n], q), PSinv, q);
        free(conv);
    }
}

/* C: [2][ell+K][N] evaluation form on the level's extended basis -> out [2][ell-1][N] evaluation form. */
static void moddown_merged_eval(uint64_t* C, uint64_t* out, const orc_level* v) {
    const orc_params* p = &v->p;
    size_t N = (size_t)1 << p->logN;
    uint32_t ell = p->L, D = ell + p->K;
    limbs_ntt(C, p, 0, D, 2, D, 1);
    for (uint32_t t = 0; t < 2; t++)
        orc_moddown_merged(C + (size_t)t * D * N, out + (size_t)t * (ell - 1) * N, p->logN, ell, p->K, p->primes);
    limbs_ntt(out, p, 0, ell - 1, 2, ell - 1, 0);
}

/* HMult + relinearisation + rescale with the merged division: level ell in, level ell-1 out.
 *   c' = inner product of the extended digits of d2 = a1*a2 with evk          ([2][ell+K][N]);
 *   C_t = c'_t + P * d_t on the q-limbs (d_0 = b1*b2, d_1 = a1*b2 + a2*b1), C_t = c'_t on the special limbs;
 *   out_t = NTT(ModDownMerged(INTT(C_t))).
 * (ModDown(c') + d = ModDown(c' + P*d) exactly, so this is HMult+relin with its ModDown and the
 * following rescale replaced by one division by P*q_{ell-1}.) */
void orc_hmult_relin_rescale_level(const uint64_t* ct1, const uint64_t* ct2, const uint64_t* evk, uint64_t* out,
                                   uint32_t ell, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                                   const uint64_t* primes, const uint64_t* psi) {
    orc_level v;
    level_open(&v, ell, logN, L, K, dnum, primes, psi);
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K;
    uint64_t* kc = level_key(&v, evk, L);
    uint64_t* d2 = (uint64_t*)malloc(sizeof(uint64_t) * ell * N);
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * v.p.dnum * D * N);
    uint64_t* C = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    for (uint32_t i = 0; i < ell; i++) {
        const uint64_t *a1 = ct1 + ((size_t)ell + i) * N, *a2 = ct2 + ((size_t)ell + i) * N;
        for (size_t n = 0; n < N; n++) d2[(size_t)i * N + n] = orc_mulmod(a1[n], a2[n], primes[i]);
    }
    decompose_extend_level(d2, dhat, &v);
    key_inner_product(dhat, kc, C, &v.p, 1);
    for (uint32_t i = 0; i < ell; i++) {
        uint64_t m = primes[i], Pm = 1;
        for (uint32_t k = 0; k < K; k++) Pm = orc_mulmod(Pm, primes[L + k] % m, m);
        const uint64_t *b1 = ct1 + (size_t)i * N, *a1 = ct1 + ((size_t)ell + i) * N;
        const uint64_t *b2 = ct2 + (size_t)i * N, *a2 = ct2 + ((size_t)ell + i) * N;
        uint64_t *C0 = C + (size_t)i * N, *C1 = C + ((size_t)D + i) * N;
        for (size_t n = 0; n < N; n++) {
            uint64_t d0 = orc_mulmod(b1[n], b2[n], m);
            uint64_t d1 = orc_addmod(orc_mulmod(a1[n], b2[n], m), orc_mulmod(a2[n], b1[n], m), m);
            C0[n] = orc_addmod(C0[n], orc_mulmod(Pm, d0, m), m);
            C1[n] = orc_addmod(C1[n], orc_mulmod(Pm, d1, m), m);
        }
    }
    moddown_merged_eval(C, out, &v);
    free(kc);
    free(d2);
    free(dhat);
    free(C);
    level_close(&v);
}

/* Double-hoisted rotate-multiply-accumulate followed by a rescale, with the merged division:
 *   C_t as in orc_hrot_dh_mac_level, plus P * sum_r pt_r * sigma_{g_r}(b) added to C_0 on the q-limbs
 *   (ModDown(C) + x = ModDown(C + P*x) exactly);   out_t = NTT(ModDownMerged(INTT(C_t))):  [2][ell-1][N]. */
void orc_hrot_dh_mac_rescale_level(const uint64_t* ct, uint32_t n_rot, const uint32_t* galois,
                                   const uint64_t* const* rk, const uint64_t* pt, uint64_t* out, uint32_t ell,
                                   uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, const uint64_t* primes,
                                   const uint64_t* psi) {
    orc_level v;
    level_open(&v, ell, logN, L, K, dnum, primes, psi);
    size_t N = (size_t)1 << logN;
    uint32_t D = ell + K;
    uint64_t* dhat = (uint64_t*)malloc(sizeof(uint64_t) * v.p.dnum * D * N);
    uint64_t* cp = (uint64_t*)malloc(sizeof(uint64_t) * 2 * D * N);
    uint64_t* C = (uint64_t*)calloc(2 * D * N, sizeof(uint64_t));
    uint64_t* sb = (uint64_t*)malloc(sizeof(uint64_t) * N);
    decompose_extend_level(ct + (size_t)ell * N, dhat, &v);
    for (uint32_t r = 0; r < n_rot; r++) {
        uint64_t* kc = level_key(&v, rk[r], L);
        key_inner_product(dhat, kc, cp, &v.p, galois[r]);
        free(kc);
        for (uint32_t t = 0; t < 2; t++)
            for (uint32_t i = 0; i < D; i++) {
                uint64_t m = v.vprimes[i];
                const uint64_t* ptr = pt + ((size_t)r * D + i) * N;
                const uint64_t* src = cp + ((size_t)t * D + i) * N;
                uint64_t* dst = C + ((size_t)t * D + i) * N;
                for (size_t n = 0; n < N; n++) dst[n] = orc_addmod(dst[n], orc_mulmod(ptr[n], src[n], m), m);
            }
        for (uint32_t i = 0; i < ell; i++) {
            uint64_t m = primes[i], Pm = 1;
            for (uint32_t k = 0; k < K; k++) Pm = orc_mulmod(Pm, primes[L + k] % m, m);
            orc_automorph_eval(ct + (size_t)i * N, sb, logN, galois[r]);
            const uint64_t* ptr = pt + ((size_t)r * D + i) * N;
            uint64_t* dst = C + (size_t)i * N;
            for (size_t n = 0; n < N; n++)
                dst[n] = orc_addmod(dst[n], orc_mulmod(Pm, orc_mulmod(ptr[n], sb[n], m), m), m);
        }
    }
    moddown_merged_eval(C, out, &v);
    free(dhat);
    free(cp);
    free(C);
    free(sb);
    level_close(&v);
}

/* --------------------------------------------------------- harness: key gen */
/* Switching key from s to s' under the RNS gadget (P on digit j's own limbs):
 *   key[j][1][i] = a_j[i]                                   (uniform, evaluation form, given)
 *   key[j][0][i] = -a_j[i]*s^[i] + e^_j[i] + (i in C_j ? (P mod q_i) * s'^[i] : 0)   mod prime_i
 * s_hat, sp_hat: [L+K][N] evaluation form; a: [dnum][L+K][N]; e: [dnum][N] signed small
 * coefficients (lifted to every limb and transformed here). key: [dnum][2][L+K][N]. */
void orc_make_switch_key(const uint64_t* s_hat, const uint64_t* sp_hat, const uint64_t* a, const int64_t* e,
                         uint64_t* key, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                         const uint64_t* primes, const uint64_t* psi) {
    size_t N = (size_t)1 << logN;
    uint32_t D = L + K, alpha = (L + dnum - 1) / dnum; /* as in the level functions */
    long total = (long)dnum * D;
#pragma omp parallel for schedule(dynamic)
    for (long id = 0; id < total; id++) {
        uint32_t j = (uint32_t)(id / D), i = (uint32_t)(id % D);
        uint64_t m = primes[i];
        uint64_t* eh = (uint64_t*)malloc(sizeof(uint64_t) * N);
        for (size_t n = 0; n < N; n++) {
            int64_t v = e[(size_t)j * N + n];
            eh[n] = v >= 0 ? (uint64_t)v % m : (m - ((uint64_t)(-v) % m)) % m;
        }
        orc_ntt(eh, logN, m, psi[i]);
        uint64_t Pm = 0;
        if (i >= j * alpha && i < (j + 1) * alpha) {
            Pm = 1;
            for (uint32_t k = 0; k < K; k++) Pm = orc_mulmod(Pm, primes[L + k] % m, m);
        }
        const uint64_t* aj = a + ((size_t)j * D + i) * N;
        uint64_t* k0 = key + (((size_t)j * 2 + 0) * D + i) * N;
        uint64_t* k1 = key + (((size_t)j * 2 + 1) * D + i) * N;
        for (size_t n = 0; n < N; n++) {
            uint64_t v = orc_submod(eh[n], orc_mulmod(aj[n], s_hat[(size_t)i * N + n], m), m);
            v = orc_addmod(v, orc_mulmod(Pm, sp_hat[(size_t)i * N + n], m), m);
            k0[n] = v;
            k1[n] = aj[n];
        }
        free(eh);
    }
}

/* Pointwise helpers for the decrypt-and-bound checks (evaluation form, one limb each). */
void orc_pointwise_mul(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t N, uint64_t m) {
    for (size_t n = 0; n < N; n++) out[n] = orc_mulmod(a[n], b[n], m);
}
void orc_pointwise_add(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t N, uint64_t m) {
    for (size_t n = 0; n < N; n++) out[n] = orc_addmod(a[n], b[n], m);
}
void orc_pointwise_sub(const uint64_t* a, const uint64_t* b, uint64_t* out, size_t N, uint64_t m) {
    for (size_t n = 0; n < N; n++) out[n] = orc_submod(a[n], b[n], m);
}
