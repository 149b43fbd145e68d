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
#ifndef INV_STRIDED_HALF_EXCHANGE
#define INV_STRIDED_HALF_EXCHANGE 1
#endif
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

    // ---- forward contiguous pass: x in layout CA (row r of the limb) -> 8 stages -> layout CB.
    // TW supplies the twiddle of stage u for the pair whose first word has index w in the row: get(u, w).
    template <class TW>
    static __device__ __forceinline__ void fwd_contig_with(T (&x)[16], u64* l, u32 e0, const TW& tw, const Mod& m) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int d = 8 >> u;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                // the strided pass leaves values below 8q: even stages reduce, odd stages run on inputs below 6q
                if (u & 1) AR::template bfly_fwd<false>(x[k], x[k + d], tw.get(u, (u32)k * 16 + e0), m);
                else AR::template bfly_fwd<true>(x[k], x[k + d], tw.get(u, (u32)k * 16 + e0), m);
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
                if (u & 1) AR::template bfly_fwd<false>(x[k], x[k + d], tw.get(u, e0 * 16 + (u32)k), m);
                else AR::template bfly_fwd<true>(x[k], x[k + d], tw.get(u, e0 * 16 + (u32)k), m);
            }
        }
    }
    // twiddles from the tables in global memory: stage u of the pass uses W[2^(A+u) + r*2^u + (w >> (8-u))]
    struct GlobalTw {
        const u64* ti;
        const double* tf;
        u32 r, N;
        __device__ __forceinline__ typename AR::Tw get(int u, u32 w) const {
            return AR::tw(ti, tf, (1u << (A + u)) + (r << u) + (w >> (8 - u)), N, false);
        }
    };
    static __device__ __forceinline__ void fwd_contig(T (&x)[16], u64* l, u32 e0, u32 r, const u64* ti,
                                                      const double* tf, u32 N, const Mod& m) {
        fwd_contig_with(x, l, e0, GlobalTw{ti, tf, r, N}, m);
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
            if constexpr (A == 8 && INV_STRIDED_HALF_EXCHANGE) {
                // N = 2^16: the exchange is a 16 x 16 transpose between the 16 lanes of a column (lane r1 register k <->
                // lane k register r1), done in two halves of eight registers through a buffer of half the size: the
                // lanes with r1 < 8 find all their words in the first half, the others in the second.  16 KiB of LDS
                // per workgroup instead of 32 lets the registers, not the LDS, set the number of resident workgroups.
                T y[16];
#pragma unroll
                for (int k = 0; k < 8; k++) lds[(r1 * 8 + k) * 16 + c] = AR::to_raw(AR::round_reduce(x[k], m));
                __syncthreads();
                if (r1 < 8) {
#pragma unroll
                    for (int k = 0; k < 16; k++) y[k] = AR::from_raw(lds[(k * 8 + r1) * 16 + c]);
                }
                __syncthreads();
#pragma unroll
                for (int k = 0; k < 8; k++) lds[(r1 * 8 + k) * 16 + c] = AR::to_raw(AR::round_reduce(x[k + 8], m));
                __syncthreads();
                if (r1 >= 8) {
#pragma unroll
                    for (int k = 0; k < 16; k++) y[k] = AR::from_raw(lds[(k * 8 + r1 - 8) * 16 + c]);
                }
#pragma unroll
                for (int k = 0; k < 16; k++) x[k] = y[k];
            } else {
#pragma unroll
                for (int k = 0; k < 16; k++) lds[(r1 * 16 + k) * TC + c] = AR::to_raw(AR::round_reduce(x[k], m));
                __syncthreads();
#pragma unroll
                for (int k = 0; k < 16; k++) x[k] = AR::from_raw(lds[k * 256 + tid]);
            }
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
