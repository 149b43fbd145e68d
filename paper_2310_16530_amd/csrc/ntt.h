// Two-pass negacyclic NTT / inverse NTT over limb batches (paper, Section 2: the NTT is one of
// the two major, memory-bound kernels of the RNS-CKKS GPU library).
//
// N = 2^logN = R1 * 256 with R1 = 2^A rows (A = logN - 8).  A limb is viewed as an R1 x 256
// matrix in row-major order.  The forward transform (natural order in, bit-reversed order out)
// runs its first A butterfly stages down the columns ("strided" pass) and the last 8 stages
// inside each 256-word row ("contiguous" pass); the inverse runs the mirror image.  Every
// workgroup of 256 threads owns 4096 words; each thread keeps 16 words in registers, performs up
// to 4 radix-2 stages on them, exchanges through LDS once and performs the remaining stages.
// Global accesses are segments of >= 128 contiguous bytes.
//
// Twiddle convention: W[k] = psi^bitrev(k), k < N, so that the stage with `g` groups uses
// W[g + i] for group i; the inverse uses the same layout built from psi^-1.
#pragma once
#include "modarith.h"

struct PrimeConst {
    u64 q;        // the prime
    u64 qneg;     // -q^-1 mod 2^64
    u64 r2;       // 2^128 mod q
    u64 ninv;     // N^-1 mod q
    u64 ninv_p;   // its Shoup companion
    u64 wlast;    // psi^-bitrev(1) * N^-1 mod q  (twiddle of the last inverse stage, pre-scaled)
    u64 wlast_p;  // its Shoup companion
    u64 pad;
};

struct NttTables {
    const u64* tw;         // [n_primes][4][N]: forward w, forward w', inverse w, inverse w'
    const PrimeConst* pc;  // [n_primes]
    u32 logN;
};

// Which limbs of a buffer a launch works on.  Job `id` -> group g = id / cnt, l' = id % cnt,
// limb-in-group l = first + l' (plus alpha if skip_alpha and l >= (g % dnum) * alpha, which
// skips the limbs owned by digit g % dnum); word offset (g*gs + l) * N; prime prime_base + l.
struct LimbMap {
    u32 cnt, gs, first, prime_base, skip_alpha, dnum;
};

__device__ __forceinline__ void resolve_limb(const LimbMap& m, u32 id, u32& limb_off, u32& prime) {
    u32 g = id / m.cnt;
    u32 l = m.first + id % m.cnt;
    if (m.skip_alpha) {
        u32 j = g % m.dnum;
        if (l >= j * m.skip_alpha) l += m.skip_alpha;
    }
    limb_off = g * m.gs + l;
    prime = m.prime_base + l;
}

__device__ __forceinline__ void bfly_fwd(u64& X, u64& Y, u64 w, u64 wp, u64 q, u64 q2) {
    u64 x = X >= q2 ? X - q2 : X;
    u64 t = mul_shoup_lazy(Y, w, wp, q);
    X = x + t;
    Y = x - t + q2;
}

__device__ __forceinline__ void bfly_inv(u64& X, u64& Y, u64 w, u64 wp, u64 q, u64 q2) {
    u64 s = X + Y;
    u64 d = X - Y + q2;
    X = s >= q2 ? s - q2 : s;
    Y = mul_shoup_lazy(d, w, wp, q);
}

#define NTT_LDS_CHUNK 272  // 256 words + one pad word per 16
__device__ __forceinline__ u32 pad16(u32 e) { return e + (e >> 4); }

// ------------------------------------------------------------------ forward, strided pass
template <int A>
__global__ __launch_bounds__(256) void ntt_fwd_strided_kernel(u64* __restrict__ data, LimbMap map, NttTables tb) {
    constexpr int R1 = 1 << A, TC = 4096 / R1, RB = R1 / 16, TILES = R1 / 16;
    __shared__ u64 lds[4096];
    const u32 N = 1u << tb.logN;
    const u32 tid = threadIdx.x;
    const u32 tile = blockIdx.x % TILES, job = blockIdx.x / TILES;
    u32 limb_off, pi;
    resolve_limb(map, job, limb_off, pi);
    u64* base = data + (size_t)limb_off * N;
    const u64* W = tb.tw + (size_t)pi * 4 * N;
    const u64* Wp = W + N;
    const u64 q = tb.pc[pi].q, q2 = 2 * q;
    const u32 c = tid % TC, r0 = tid / TC, col = tile * TC + c;

    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = base[(size_t)(k * RB + r0) * 256 + col];
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const int d = 8 >> s;
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (1u << s) + (k >> (4 - s));
            bfly_fwd(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
    if constexpr (A == 4) {
#pragma unroll
        for (int k = 0; k < 16; k++) base[(size_t)(k * RB + r0) * 256 + col] = x[k];
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) lds[k * 256 + tid] = x[k];
        __syncthreads();
        const u32 r1 = r0;
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = lds[(r1 * 16 + k) * TC + c];
#pragma unroll
        for (int s = 4; s < A; s++) {
            const int d = 1 << (A - s - 1);
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                const u32 ti = (1u << s) + ((r1 * 16 + k) >> (A - s));
                bfly_fwd(x[k], x[k + d], W[ti], Wp[ti], q, q2);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) base[(size_t)(r1 * 16 + k) * 256 + col] = x[k];
    }
}

// --------------------------------------------------------------- forward, contiguous pass
// Input values in [0, 4q); output canonical.
template <int A>
__global__ __launch_bounds__(256) void ntt_fwd_contig_kernel(u64* __restrict__ data, LimbMap map, NttTables tb) {
    constexpr int R1 = 1 << A, TILES = R1 / 16;
    __shared__ u64 lds[16 * NTT_LDS_CHUNK];
    const u32 N = 1u << tb.logN;
    const u32 tid = threadIdx.x;
    const u32 tile = blockIdx.x % TILES, job = blockIdx.x / TILES;
    u32 limb_off, pi;
    resolve_limb(map, job, limb_off, pi);
    const u64* W = tb.tw + (size_t)pi * 4 * N;
    const u64* Wp = W + N;
    const u64 q = tb.pc[pi].q, q2 = 2 * q;
    const u32 e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    u64* ptr = data + (size_t)limb_off * N + (size_t)r * 256;
    u64* l = lds + ch * NTT_LDS_CHUNK;

    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = ptr[k * 16 + e0];
#pragma unroll
    for (int u = 0; u < 4; u++) {
        const int d = 8 >> u;
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (1u << (A + u)) + (r << u) + (k >> (4 - u));
            bfly_fwd(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
#pragma unroll
    for (int k = 0; k < 16; k++) l[pad16(k * 16 + e0)] = x[k];
    __syncthreads();
    const u32 e1 = e0;
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = l[pad16(e1 * 16 + k)];
#pragma unroll
    for (int u = 4; u < 8; u++) {
        const int d = 8 >> (u - 4);
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (1u << (A + u)) + (r << u) + ((e1 * 16 + k) >> (8 - u));
            bfly_fwd(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) l[pad16(e1 * 16 + k)] = csub(csub(x[k], q2), q);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) ptr[k * 16 + e0] = l[pad16(k * 16 + e0)];
}

// --------------------------------------------------------------- inverse, contiguous pass
// Input canonical (evaluation form); output in [0, 2q).
template <int A>
__global__ __launch_bounds__(256) void ntt_inv_contig_kernel(u64* __restrict__ data, LimbMap map, NttTables tb) {
    constexpr int R1 = 1 << A, TILES = R1 / 16;
    __shared__ u64 lds[16 * NTT_LDS_CHUNK];
    const u32 N = 1u << tb.logN;
    const u32 tid = threadIdx.x;
    const u32 tile = blockIdx.x % TILES, job = blockIdx.x / TILES;
    u32 limb_off, pi;
    resolve_limb(map, job, limb_off, pi);
    const u64* W = tb.tw + (size_t)pi * 4 * N + 2 * (size_t)N;
    const u64* Wp = W + N;
    const u64 q = tb.pc[pi].q, q2 = 2 * q;
    const u32 e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    u64* ptr = data + (size_t)limb_off * N + (size_t)r * 256;
    u64* l = lds + ch * NTT_LDS_CHUNK;

    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) l[pad16(k * 16 + e0)] = ptr[k * 16 + e0];
    __syncthreads();
    const u32 e1 = e0;
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = l[pad16(e1 * 16 + k)];
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const int d = 1 << v;
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (N >> (v + 1)) + ((r * 256 + e1 * 16 + k) >> (v + 1));
            bfly_inv(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) l[pad16(e1 * 16 + k)] = x[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = l[pad16(k * 16 + e0)];
#pragma unroll
    for (int v = 4; v < 8; v++) {
        const int d = 1 << (v - 4);
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (N >> (v + 1)) + ((r * 256 + k * 16) >> (v + 1));
            bfly_inv(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
#pragma unroll
    for (int k = 0; k < 16; k++) ptr[k * 16 + e0] = x[k];
}

// ------------------------------------------------------------------ inverse, strided pass
// Input in [0, 2q); output canonical, scaled by N^-1 (natural-order coefficients).
template <int A>
__global__ __launch_bounds__(256) void ntt_inv_strided_kernel(u64* __restrict__ data, LimbMap map, NttTables tb) {
    constexpr int R1 = 1 << A, TC = 4096 / R1, RB = R1 / 16, TILES = R1 / 16;
    __shared__ u64 lds[4096];
    const u32 N = 1u << tb.logN;
    const u32 tid = threadIdx.x;
    const u32 tile = blockIdx.x % TILES, job = blockIdx.x / TILES;
    u32 limb_off, pi;
    resolve_limb(map, job, limb_off, pi);
    u64* base = data + (size_t)limb_off * N;
    const u64* W = tb.tw + (size_t)pi * 4 * N + 2 * (size_t)N;
    const u64* Wp = W + N;
    const PrimeConst pc = tb.pc[pi];
    const u64 q = pc.q, q2 = 2 * q;
    const u32 c = tid % TC, r0 = tid / TC, col = tile * TC + c;

    u64 x[16];
    if constexpr (A > 4) {
        const u32 r1 = r0;
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = base[(size_t)(r1 * 16 + k) * 256 + col];
#pragma unroll
        for (int w = 0; w < A - 4; w++) {
            const int d = 1 << w;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                const u32 ti = (N >> (9 + w)) + ((r1 * 16 + k) >> (w + 1));
                bfly_inv(x[k], x[k + d], W[ti], Wp[ti], q, q2);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) lds[(r1 * 16 + k) * TC + c] = x[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = lds[k * 256 + tid];
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = base[(size_t)(k * RB + r0) * 256 + col];
    }
#pragma unroll
    for (int w = A - 4; w < A - 1; w++) {
        const int d = 1 << (w - A + 4);
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if (k & d) continue;
            const u32 ti = (1u << (A - 1 - w)) + (k >> (w - A + 5));
            bfly_inv(x[k], x[k + d], W[ti], Wp[ti], q, q2);
        }
    }
    // last stage (one group, twiddle index 1) merged with the factor N^-1
#pragma unroll
    for (int k = 0; k < 8; k++) {
        u64 s = x[k] + x[k + 8];
        u64 d = x[k] - x[k + 8] + q2;
        x[k] = mul_shoup(s, pc.ninv, pc.ninv_p, q);
        x[k + 8] = mul_shoup(d, pc.wlast, pc.wlast_p, q);
    }
#pragma unroll
    for (int k = 0; k < 16; k++) base[(size_t)(k * RB + r0) * 256 + col] = x[k];
}
