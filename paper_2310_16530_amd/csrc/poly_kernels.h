// Element-parallel kernels of the key-switch path: fast base conversion (ModUp / ModDown, the
// second major kernel named in the paper's Section 2), the key inner product, the tensor
// product, the Galois automorphism and the final combine.  One thread per coefficient (or
// evaluation slot); consecutive threads touch consecutive words of a limb.
#pragma once
#include "ntt.h"

struct ShoupConst {
    u64 w, wp;
};

struct ConvTables {
    const PrimeConst* pc;          // [D]
    const ShoupConst* up_hatinv;   // [L]       [(Q_j/q_i)^-1]_{q_i} for i in digit j
    const u64* up_chat;            // [L][D]    (Q_j/q_i) * 2^64 mod m_t  (0 where t is in the digit)
    const ShoupConst* dn_hatinv;   // [K]       [(P/p_k)^-1]_{p_k}
    const u64* dn_chat;            // [K][L]    (P/p_k) * 2^64 mod q_i
    const ShoupConst* pinv;        // [L]       P^-1 mod q_i
};

// slot j of sigma_g(f) in evaluation form reads slot perm(j) of f
__device__ __forceinline__ u32 eval_perm(u32 j, u32 g, u32 logN) {
    const u32 two_n_mask = (2u << logN) - 1;
    u32 e = (g * (2 * (__brev(j) >> (32 - logN)) + 1)) & two_n_mask;
    return __brev((e - 1) >> 1) >> (32 - logN);
}

// ------------------------------------------------------------------------------- ModUp
// in [b][L][N] coeff -> out [b][dnum][D][N].  grid (N/256, dnum, batch).
template <int ALPHA>
__global__ __launch_bounds__(256) void modup_kernel(const u64* __restrict__ in, u64* __restrict__ out, ConvTables ct,
                                                    u32 logN, u32 L, u32 D, u32 dnum, int write_own) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, j = blockIdx.y, b = blockIdx.z;
    const u64* src = in + ((size_t)b * L + (size_t)j * ALPHA) * N + n;
    u64* dst = out + ((size_t)b * dnum + j) * D * N + n;
    u64 y[ALPHA];
#pragma unroll
    for (int ii = 0; ii < ALPHA; ii++) {
        const u32 i = j * ALPHA + ii;
        const u64 x = src[(size_t)ii * N];
        if (write_own) dst[(size_t)i * N] = x;
        const ShoupConst h = ct.up_hatinv[i];
        y[ii] = mul_shoup(x, h.w, h.wp, ct.pc[i].q);
    }
    const u64* chat = ct.up_chat + (size_t)j * ALPHA * D;
    for (u32 t = 0; t < D; t++) {
        if (t >= j * ALPHA && t < (j + 1) * ALPHA) continue;
        u128w acc = {0, 0};
#pragma unroll
        for (int ii = 0; ii < ALPHA; ii++) mac128(acc, y[ii], chat[(size_t)ii * D + t]);
        const PrimeConst pc = ct.pc[t];
        dst[(size_t)t * N] = redc(acc, pc.q, pc.qneg);
    }
}

// ----------------------------------------------------------------------------- ModDown
// in [g][D][N] coeff.  FUSE = true : out [g][L][N] = (in_i - conv_i) * P^-1      (full ModDown)
//                       FUSE = false: out [g][L][N] = conv_i                      (conversion only)
// grid (N/256, groups).
template <int KK, bool FUSE>
__global__ __launch_bounds__(256) void moddown_kernel(const u64* __restrict__ in, u64* __restrict__ out, ConvTables ct,
                                                      u32 logN, u32 L, u32 D) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
    const u64* src = in + (size_t)g * D * N + n;
    u64* dst = out + (size_t)g * L * N + n;
    u64 y[KK];
#pragma unroll
    for (int k = 0; k < KK; k++) {
        const ShoupConst h = ct.dn_hatinv[k];
        y[k] = mul_shoup(src[(size_t)(L + k) * N], h.w, h.wp, ct.pc[L + k].q);
    }
    for (u32 i = 0; i < L; i++) {
        u128w acc = {0, 0};
#pragma unroll
        for (int k = 0; k < KK; k++) mac128(acc, y[k], ct.dn_chat[(size_t)k * L + i]);
        const PrimeConst pc = ct.pc[i];
        u64 conv = redc(acc, pc.q, pc.qneg);
        if (FUSE) {
            const ShoupConst pi = ct.pinv[i];
            conv = mul_shoup(submod(src[(size_t)i * N], conv, pc.q), pi.w, pi.wp, pc.q);
        }
        dst[(size_t)i * N] = conv;
    }
}

// ------------------------------------------------------------------- key inner product
#define CKKS_ROT_CHUNK 8
struct KeyPtrs {
    const u64* key[CKKS_ROT_CHUNK];
    u32 galois[CKKS_ROT_CHUNK];
};

// c'[g][t][i][n] = sum_j dh[g*dh_stride + j][i][perm_g(n)] * key_g[j][t][i][n].
// grid (N/256, D, groups).  PER_GROUP_KEY: keys/galois taken from kp[g], digits shared (dh_group_stride 0).
template <bool PER_GROUP_KEY>
__global__ __launch_bounds__(256) void inner_product_kernel(const u64* __restrict__ dh, size_t dh_group_stride,
                                                            KeyPtrs kp, u64* __restrict__ cp, const PrimeConst* pcs,
                                                            u32 logN, u32 D, u32 dnum) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y, g = blockIdx.z;
    const u64* key = kp.key[PER_GROUP_KEY ? g : 0];
    u32 src_n = n;
    if (PER_GROUP_KEY) {
        const u32 gal = kp.galois[g];
        if (gal != 1) src_n = eval_perm(n, gal, logN);
    }
    const u64* d = dh + (size_t)g * dh_group_stride + (size_t)i * N + src_n;
    const u64* k = key + (size_t)i * N + n;
    u128w a0 = {0, 0}, a1 = {0, 0};
    for (u32 j = 0; j < dnum; j++) {
        const u64 dv = d[(size_t)j * D * N];
        mac128(a0, dv, k[((size_t)j * 2 + 0) * D * N]);
        mac128(a1, dv, k[((size_t)j * 2 + 1) * D * N]);
    }
    const PrimeConst pc = pcs[i];
    u64* o = cp + ((size_t)g * 2 * D + i) * N + n;
    o[0] = reduce128(a0, pc.q, pc.qneg, pc.r2);
    o[(size_t)D * N] = reduce128(a1, pc.q, pc.qneg, pc.r2);
}

// ------------------------------------------------------------ preparation (evaluation form)
// Each writes the evaluation-form polynomial that is to be switched into x [b][L][N] and into
// the own-digit slots of dt [b][dnum][D][N] (digit i/alpha, limb i).  grid (N/256, L, batch).
enum PrepMode { PREP_COPY = 0, PREP_TENSOR_D2 = 1, PREP_ROT_A = 2 };

template <int MODE>
__global__ __launch_bounds__(256) void prep_kernel(const u64* __restrict__ in1, const u64* __restrict__ in2,
                                                   u64* __restrict__ x, u64* __restrict__ dt, const PrimeConst* pcs,
                                                   u32 logN, u32 L, u32 D, u32 dnum, u32 alpha, u32 galois) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y, b = blockIdx.z;
    u64 v;
    if (MODE == PREP_COPY) {
        v = in1[((size_t)b * L + i) * N + n];
    } else if (MODE == PREP_TENSOR_D2) {
        const PrimeConst pc = pcs[i];
        const u64 a1 = in1[(((size_t)b * 2 + 1) * L + i) * N + n];
        const u64 a2 = in2[(((size_t)b * 2 + 1) * L + i) * N + n];
        v = mulmod_var(a1, a2, pc.q, pc.qneg, pc.r2);
    } else {
        v = in1[(((size_t)b * 2 + 1) * L + i) * N + eval_perm(n, galois, logN)];
    }
    x[((size_t)b * L + i) * N + n] = v;
    const u32 j = i / alpha;
    dt[(((size_t)b * dnum + j) * D + i) * N + n] = v;
}

// ------------------------------------------------------------------------ final combine
// ks_t[i] = (c'_t[i] - convh_t[i]) * P^-1 mod q_i   (all evaluation form), then
//   FIN_KS     : out[g][t][i] = ks
//   FIN_HMULT  : out = ks + (t == 0 ? b1*b2 : a1*b2 + a2*b1)
//   FIN_HROT   : out = ks + (t == 0 ? sigma_g(b) : 0)
//   FIN_HOISTED: out[t][i] (+)= sum_{r < n_rot} pt_r[i] * (ks_r + (t == 0 ? sigma_{g_r}(b) : 0))
// cp [g][2][D][N], cv [g][2][L][N].  grid (N/256, L, groups*2) except FIN_HOISTED: (N/256, L, 2).
enum FinalMode { FIN_KS = 0, FIN_HMULT = 1, FIN_HROT = 2, FIN_HOISTED = 3 };

struct FinalArgs {
    const u64* cp;
    const u64* cv;
    const u64* ct1;  // HMULT: ct1; HROT / HOISTED: ct
    const u64* ct2;  // HMULT: ct2
    const u64* pt;   // HOISTED: plaintexts of this chunk [n_rot][L][N]
    u64* out;
    u32 galois[CKKS_ROT_CHUNK];
    u32 n_rot;
    u32 accumulate;  // HOISTED: add to what out already holds
};

template <int MODE>
__global__ __launch_bounds__(256) void final_kernel(FinalArgs a, ConvTables ct, u32 logN, u32 L, u32 D) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
    const PrimeConst pc = ct.pc[i];
    const ShoupConst pinv = ct.pinv[i];
    const u64 q = pc.q;
    if (MODE == FIN_HOISTED) {
        const u32 t = blockIdx.z;
        u128w acc = {0, 0};
        for (u32 r = 0; r < a.n_rot; r++) {
            const u64 c = a.cp[(((size_t)r * 2 + t) * D + i) * N + n];
            const u64 v = a.cv[(((size_t)r * 2 + t) * L + i) * N + n];
            u64 ks = mul_shoup(submod(c, v, q), pinv.w, pinv.wp, q);
            if (t == 0) ks = addmod(ks, a.ct1[(size_t)i * N + eval_perm(n, a.galois[r], logN)], q);
            mac128(acc, ks, a.pt[((size_t)r * L + i) * N + n]);
        }
        u64 res = reduce128(acc, q, pc.qneg, pc.r2);
        u64* o = a.out + ((size_t)t * L + i) * N + n;
        if (a.accumulate) res = addmod(res, *o, q);
        *o = res;
        return;
    }
    const u32 g = blockIdx.z >> 1, t = blockIdx.z & 1;
    const u64 c = a.cp[(((size_t)g * 2 + t) * D + i) * N + n];
    const u64 v = a.cv[(((size_t)g * 2 + t) * L + i) * N + n];
    u64 ks = mul_shoup(submod(c, v, q), pinv.w, pinv.wp, q);
    if (MODE == FIN_HMULT) {
        const size_t o0 = (((size_t)g * 2 + 0) * L + i) * N + n, o1 = (((size_t)g * 2 + 1) * L + i) * N + n;
        const u64 b1 = a.ct1[o0], a1 = a.ct1[o1], b2 = a.ct2[o0], a2 = a.ct2[o1];
        u128w acc = {0, 0};
        if (t == 0) {
            mac128(acc, b1, b2);
        } else {
            mac128(acc, a1, b2);
            mac128(acc, a2, b1);
        }
        ks = addmod(ks, reduce128(acc, q, pc.qneg, pc.r2), q);
    } else if (MODE == FIN_HROT) {
        if (t == 0) ks = addmod(ks, a.ct1[(((size_t)g * 2) * L + i) * N + eval_perm(n, a.galois[0], logN)], q);
    }
    a.out[(((size_t)g * 2 + t) * L + i) * N + n] = ks;
}

// ------------------------------------------------------------------------ automorphism
// [groups][n_limbs][N] -> same shape.  grid (N/256, n_limbs, batch).
__global__ __launch_bounds__(256) void automorph_eval_kernel(const u64* __restrict__ in, u64* __restrict__ out, u32 logN,
                                                             u32 n_limbs, u32 galois) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x;
    const size_t limb = ((size_t)blockIdx.z * n_limbs + blockIdx.y) * N;
    out[limb + n] = in[limb + eval_perm(n, galois, logN)];
}

// coefficient form, as a gather: out[u] = +-in[t] with t*g = u (mod 2N) or t*g = u + N (mod 2N)
__global__ __launch_bounds__(256) void automorph_coeff_kernel(const u64* __restrict__ in, u64* __restrict__ out,
                                                              const PrimeConst* pcs, u32 logN, u32 n_limbs,
                                                              u32 prime_first, u32 galois_inv) {
    const u32 N = 1u << logN;
    const u32 u = blockIdx.x * 256 + threadIdx.x;
    const size_t limb = ((size_t)blockIdx.z * n_limbs + blockIdx.y) * N;
    const u64 q = pcs[prime_first + blockIdx.y].q;
    const u32 tp = (u * galois_inv) & (2 * N - 1);
    u64 v;
    if (tp < N) {
        v = in[limb + tp];
    } else {
        v = in[limb + tp - N];
        v = v ? q - v : 0;
    }
    out[limb + u] = v;
}
