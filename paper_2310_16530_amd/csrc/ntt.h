// Building blocks of the two-pass negacyclic NTT / inverse NTT (paper, Section 2: the NTT is one
// of the two major, memory-bound kernels of the RNS-CKKS GPU library).
//
// N = 2^logN = R1 * 256 with R1 = 2^A rows (A = logN - 8).  A limb is viewed as an R1 x 256
// row-major matrix.  The forward transform (natural order in, bit-reversed order out) runs its
// first A butterfly stages down the columns ("strided" pass) and the last 8 stages inside each
// 256-word row ("contiguous" pass); the inverse runs the mirror image.  A workgroup of 256
// threads owns 4096 words; a thread keeps 16 words in registers, performs up to 4 radix-2 stages
// on them, exchanges through LDS once and performs the remaining stages.  The passes are written
// as device functions over the register array so that producers (base conversion, tensor
// product, automorphism) and consumers (key inner product, final combine) fuse into them.
//
// Register layouts of the 16 words x[k] of thread `tid`:
//   strided pass, tile = all R1 rows x TC = 4096/R1 columns, c = tid % TC, r0 = tid / TC:
//     layout SA: row k*(R1/16) + r0, column c        layout SB: row r0*16 + k, column c
//   contiguous pass, tile = 16 rows, e0 = tid % 16, ch = tid / 16 (row within the tile):
//     layout CA: word k*16 + e0 of the row            layout CB: word e0*16 + k of the row
// CA and SA/SB are the coalesced layouts (>= 128 contiguous bytes per 16 lanes).
//
// Twiddle convention: W[k] = psi^bitrev(k), k < N: the stage with g groups uses W[g + i] for
// group i; the inverse uses the same layout built from psi^-1.
#pragma once
#include "modarith.h"

#define NTT_LDS_WORDS (16 * 272)  // 16 rows of 256 words + one pad word per 16
__device__ __forceinline__ u32 pad16(u32 e) { return e + (e >> 4); }

// In the contiguous pass the 16 lanes that own a row are part of one wavefront and no other
// wavefront touches that row's LDS slice, so exchanges need no workgroup barrier: LDS operations
// of one wavefront execute in issue order; the fence keeps the compiler from reordering them.
__device__ __forceinline__ void row_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <class AR, int A>
struct NttCore {
    typedef typename AR::T T;
    typedef typename AR::Mod Mod;
    static constexpr int R1 = 1 << A, TC = 4096 / R1, RB = R1 / 16;

    // ---- forward strided pass: x in layout SA -> all A stages -> layout SB (A > 4) or SA (A == 4)
    static __device__ __forceinline__ void fwd_strided(T (&x)[16], u64* lds, u32 tid, const u64* ti, const double* tf,
                                                       u32 N, const Mod& m) {
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int d = 8 >> s;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                // inputs are canonical: below 3q, 5q, 7q before stages 1, 2, 3, so only stage 3 reduces first
                if (s == 3) AR::template bfly_fwd<true>(x[k], x[k + d], AR::tw(ti, tf, (1u << s) + (k >> (4 - s)), N, false), m);
                else AR::template bfly_fwd<false>(x[k], x[k + d], AR::tw(ti, tf, (1u << s) + (k >> (4 - s)), N, false), m);
            }
        }
        if constexpr (A > 4) {
            const u32 c = tid % TC, r1 = tid / TC;
#pragma unroll
            for (int k = 0; k < 16; k++) lds[k * 256 + tid] = AR::to_raw(AR::round_reduce(x[k], m));
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 16; k++) x[k] = AR::from_raw(lds[(r1 * 16 + k) * TC + c]);
#pragma unroll
            for (int s = 4; s < A; s++) {
                const int d = 1 << (A - s - 1);
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    if (k & d) continue;
                    // below 6q after stage 3: from here odd stages reduce, even stages run on inputs below 6q
                    if (s & 1) AR::template bfly_fwd<true>(x[k], x[k + d], AR::tw(ti, tf, (1u << s) + ((r1 * 16 + k) >> (A - s)), N, false), m);
                    else AR::template bfly_fwd<false>(x[k], x[k + d], AR::tw(ti, tf, (1u << s) + ((r1 * 16 + k) >> (A - s)), N, false), m);
                }
            }
        }
    }

    // ---- forward contiguous pass: x in layout CA (row r of the limb) -> 8 stages -> layout CB
    static __device__ __forceinline__ void fwd_contig(T (&x)[16], u64* l, u32 e0, u32 r, const u64* ti,
                                                      const double* tf, u32 N, const Mod& m) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int d = 8 >> u;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                // the strided pass leaves values below 8q: even stages reduce, odd stages run on inputs below 6q
                if (u & 1) AR::template bfly_fwd<false>(x[k], x[k + d], AR::tw(ti, tf, (1u << (A + u)) + (r << u) + (k >> (4 - u)), N, false), m);
                else AR::template bfly_fwd<true>(x[k], x[k + d], AR::tw(ti, tf, (1u << (A + u)) + (r << u) + (k >> (4 - u)), N, false), m);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) l[pad16(k * 16 + e0)] = AR::to_raw(AR::round_reduce(x[k], m));
        row_sync();
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::from_raw(l[pad16(e0 * 16 + k)]);
#pragma unroll
        for (int u = 4; u < 8; u++) {
            const int d = 8 >> (u - 4);
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                if (u & 1) AR::template bfly_fwd<false>(x[k], x[k + d],
                             AR::tw(ti, tf, (1u << (A + u)) + (r << u) + ((e0 * 16 + k) >> (8 - u)), N, false), m);
                else AR::template bfly_fwd<true>(x[k], x[k + d],
                             AR::tw(ti, tf, (1u << (A + u)) + (r << u) + ((e0 * 16 + k) >> (8 - u)), N, false), m);
            }
        }
    }

    // ---- inverse contiguous pass: x in layout CB (inverse-lazy range) -> 8 stages -> layout CA
    static __device__ __forceinline__ void inv_contig(T (&x)[16], u64* l, u32 e0, u32 r, const u64* ti,
                                                      const double* tf, u32 N, const Mod& m) {
#pragma unroll
        for (int v = 0; v < 4; v++) {
            const int d = 1 << v;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                AR::bfly_inv(x[k], x[k + d],
                             AR::tw(ti, tf, (N >> (v + 1)) + ((r * 256 + e0 * 16 + k) >> (v + 1)), N, true), m);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) l[pad16(e0 * 16 + k)] = AR::to_raw(AR::round_reduce(x[k], m));
        row_sync();
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::from_raw(l[pad16(k * 16 + e0)]);
#pragma unroll
        for (int v = 4; v < 8; v++) {
            const int d = 1 << (v - 4);
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                AR::bfly_inv(x[k], x[k + d], AR::tw(ti, tf, (N >> (v + 1)) + ((r * 256 + k * 16) >> (v + 1)), N, true),
                             m);
            }
        }
    }

    // ---- inverse strided pass: x in layout SB (A > 4) or SA (A == 4) -> all stages but the last
    //      -> layout SA.  The caller applies the last stage (pairs x[k], x[k+8]) with its scaling.
    static __device__ __forceinline__ void inv_strided_but_last(T (&x)[16], u64* lds, u32 tid, const u64* ti,
                                                                const double* tf, u32 N, const Mod& m) {
        if constexpr (A > 4) {
            const u32 c = tid % TC, r1 = tid / TC;
#pragma unroll
            for (int w = 0; w < A - 4; w++) {
                const int d = 1 << w;
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    if (k & d) continue;
                    AR::bfly_inv(x[k], x[k + d], AR::tw(ti, tf, (N >> (9 + w)) + ((r1 * 16 + k) >> (w + 1)), N, true), m);
                }
            }
#pragma unroll
            for (int k = 0; k < 16; k++) lds[(r1 * 16 + k) * TC + c] = AR::to_raw(AR::round_reduce(x[k], m));
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 16; k++) x[k] = AR::from_raw(lds[k * 256 + tid]);
        }
#pragma unroll
        for (int w = A - 4; w < A - 1; w++) {
            const int d = 1 << (w - A + 4);
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                AR::bfly_inv(x[k], x[k + d], AR::tw(ti, tf, (1u << (A - 1 - w)) + (k >> (w - A + 5)), N, true), m);
            }
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Contiguous pass with 32 lanes per 256-word row and 8 words per lane: half the registers per lane of the
// 16-word form above, for kernels that keep accumulators across several transforms (the key inner product)
// and are limited by the waves their registers allow.  A wavefront owns two rows; a 256-thread workgroup a
// tile of 8 rows.  The 8 stages run as 3 + 3 + 2 in-lane stages with two exchanges through the row's LDS
// slice (wave-local, row_sync).  Register layouts of the 8 words x[k] of lane e (word index w in the row):
//   R0: w = k*32 + e                              coalesced global access; in-lane bits 7,6,5
//   RF: w = (e/4)*32 + k*4 + e%4                  forward middle round;    in-lane bits 4,3,2
//   R2: w = e*8 + k                               in-lane bits 2,1,0
//   RI: w = (e/8)*64 + k*8 + e%8                  inverse middle round;    in-lane bits 5,4,3
// forward: R0 (stages 0-2) -> RF (stages 3-5) -> R2 (stages 6,7); inverse: R2 (0-2) -> RI (3-5) -> R0 (6,7).
// Twiddles: forward stage u of the pass uses W[2^(A+u) + r*2^u + (w >> (8-u))], inverse stage v uses
// Winv[(N >> (v+1)) + ((r*256 + w) >> (v+1))], w = row index of the pair's first word (as in NttCore).
#define NTT8_ROW_WORDS 288  // 256 words + one pad word per 8
#define NTT8_LDS_WORDS (8 * NTT8_ROW_WORDS)
__device__ __forceinline__ u32 pad8(u32 w) { return w + (w >> 3); }
__device__ __forceinline__ u32 w_r0(u32 e, u32 k) { return k * 32 + e; }
__device__ __forceinline__ u32 w_rf(u32 e, u32 k) { return ((e >> 2) << 5) | (k << 2) | (e & 3); }
__device__ __forceinline__ u32 w_r2(u32 e, u32 k) { return e * 8 + k; }
__device__ __forceinline__ u32 w_ri(u32 e, u32 k) { return ((e >> 3) << 6) | (k << 3) | (e & 7); }

enum Row8Layout { R8_R0 = 0, R8_RF = 1, R8_R2 = 2, R8_RI = 3 };
template <int LAY>
__device__ __forceinline__ u32 w_of(u32 e, u32 k) {
    return LAY == R8_R0 ? w_r0(e, k) : LAY == R8_RF ? w_rf(e, k) : LAY == R8_R2 ? w_r2(e, k) : w_ri(e, k);
}

// x from layout FROM to layout TO through the row's LDS slice; REDUCE applies the arithmetic's range
// reduction to what is written (the rounds of the transforms rely on it)
template <class AR, int FROM, int TO, bool REDUCE>
__device__ __forceinline__ void row8_exchange(typename AR::T (&x)[8], u64* l, u32 e, const typename AR::Mod& m) {
    row_sync();
#pragma unroll
    for (int k = 0; k < 8; k++) l[pad8(w_of<FROM>(e, k))] = AR::to_raw(REDUCE ? AR::round_reduce(x[k], m) : x[k]);
    row_sync();
#pragma unroll
    for (int k = 0; k < 8; k++) x[k] = AR::from_raw(l[pad8(w_of<TO>(e, k))]);
}

template <class AR, int A>
struct NttRow8 {
    typedef typename AR::T T;
    typedef typename AR::Mod Mod;

    // three (or NS) in-lane forward stages starting at pass stage U0 on layout LAY
    template <int LAY, int U0, int NS>
    static __device__ __forceinline__ void fwd_round(T (&x)[8], u32 e, u32 r, const u64* ti, const double* tf, u32 N,
                                                     const Mod& m) {
#pragma unroll
        for (int s = 0; s < NS; s++) {
            const int u = U0 + s;
            const int d = (NS == 3 ? 4 : 2) >> s;  // in-lane distance of the pair
#pragma unroll
            for (int k = 0; k < 8; k++) {
                if (k & d) continue;
                const u32 w = w_of<LAY>(e, k);
                const typename AR::Tw t = AR::tw(ti, tf, (1u << (A + u)) + (r << u) + (w >> (8 - u)), N, false);
                // values below 8q enter the pass: even stages take 4q off first, odd stages run on inputs below 6q
                if (u & 1) AR::template bfly_fwd<false>(x[k], x[k + d], t, m);
                else AR::template bfly_fwd<true>(x[k], x[k + d], t, m);
            }
        }
    }
    // x in layout R0 (row r of the limb, values as the strided pass leaves them) -> 8 stages -> layout R2
    static __device__ __forceinline__ void fwd_contig(T (&x)[8], u64* l, u32 e, u32 r, const u64* ti, const double* tf,
                                                      u32 N, const Mod& m) {
        fwd_round<R8_R0, 0, 3>(x, e, r, ti, tf, N, m);
        row8_exchange<AR, R8_R0, R8_RF, true>(x, l, e, m);
        fwd_round<R8_RF, 3, 3>(x, e, r, ti, tf, N, m);
        row8_exchange<AR, R8_RF, R8_R2, true>(x, l, e, m);
        fwd_round<R8_R2, 6, 2>(x, e, r, ti, tf, N, m);
    }

    template <int LAY, int V0, int NS, int D0>
    static __device__ __forceinline__ void inv_round(T (&x)[8], u32 e, u32 r, const u64* ti, const double* tf, u32 N,
                                                     const Mod& m) {
#pragma unroll
        for (int s = 0; s < NS; s++) {
            const int v = V0 + s;
            const int d = D0 << s;  // in-lane distance of the pair
#pragma unroll
            for (int k = 0; k < 8; k++) {
                if (k & d) continue;
                const u32 w = w_of<LAY>(e, k);
                AR::bfly_inv(x[k], x[k + d], AR::tw(ti, tf, (N >> (v + 1)) + ((r * 256 + w) >> (v + 1)), N, true), m);
            }
        }
    }
    // x in layout R2 (inverse-lazy range) -> 8 stages -> layout R0
    static __device__ __forceinline__ void inv_contig(T (&x)[8], u64* l, u32 e, u32 r, const u64* ti, const double* tf,
                                                      u32 N, const Mod& m) {
        inv_round<R8_R2, 0, 3, 1>(x, e, r, ti, tf, N, m);
        row8_exchange<AR, R8_R2, R8_RI, true>(x, l, e, m);
        inv_round<R8_RI, 3, 3, 1>(x, e, r, ti, tf, N, m);
        row8_exchange<AR, R8_RI, R8_R0, true>(x, l, e, m);
        inv_round<R8_R0, 6, 2, 2>(x, e, r, ti, tf, N, m);  // bits 6 and 7 of w are bits 1 and 2 of k
    }
};

// XCD-aware decode of a linear workgroup id.  Workgroups are handed to the 8 XCDs round-robin,
// so ids congruent modulo 8 share an L2.  Work is organised as `groups` groups of `S` instances
// that read the same tables / sources; all instances of a group get ids on one XCD, adjacent
// in dispatch order.  The grid must hold ceil(groups/8)*8*S workgroups; returns false for padding.
__device__ __forceinline__ bool xcd_decode(u32 bid, u32 S, u32 groups, u32& group, u32& inst) {
    const u32 xcd = bid & 7, pos = bid >> 3;
    inst = pos % S;
    group = (pos / S) * 8 + xcd;
    return group < groups;
}
