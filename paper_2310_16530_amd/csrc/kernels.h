// Kernels of the key-switch path.  The paper (Section 2) names the NTT and the base conversion as
// the major, memory-bound kernels and fuses several jobs into each memory load; here every
// producer and consumer of a transform is fused into one of the two NTT passes:
//
//   inv_contig_kernel   load (copy | a1*a2 | sigma_g gather) -> first inverse pass
//   inv_strided_kernel  second inverse pass -> scale by N^-1 (* base-conversion pre-factor)
//   fwd_strided_kernel  load (plain | base conversion from the digit / special limbs) -> first forward pass
//   fwd_contig_kernel   second forward pass -> canonical store
//   ks_inner_kernel     second forward pass of every extended digit -> key inner product accumulated over
//                       the digits in registers (+ P * tensor terms of HMult) -> special limbs: first inverse
//                       pass of ModDown; q-limbs, launched after the ModDown conversion: second forward pass
//                       of the converted special part -> (c' - .) * P^-1 (+ sigma_g(b)) -> result
//   ks_final_kernel     the same end of the ModDown from a stored c', for the calls whose inner product is
//                       not this kernel or is followed by a plaintext multiply-accumulate over rotations
//   dh_accum_kernel     double hoisting: plaintext products of all rotations accumulated in the extended basis
//   bsgs_mac_kernel     giant-step combinations of baby-step rotations kept in the extended basis
//   modup_kernel / moddown_kernel / automorph kernels: the stand-alone coefficient-form entry points.
//
// Levels below L, rescale and the ModDown merged with a rescale reuse these kernels on per-level tables.
//
// Every kernel picks its arithmetic per limb: FpAr for primes below 3*2^48, IntAr otherwise.
#pragma once
#include "ntt.h"

struct PinvConst {
    u64 w, wp;
    double d;
};

struct Tables {
    const u64* tw_int;         // [D][4][N]  fwd w, fwd w', inv w, inv w'
    const double* tw_fp;       // [D][2][N]  fwd w, inv w (FpAr primes only)
    const PrimeConst* pc;      // [D]
    const InvScale* sc_plain;  // [D]  N^-1
    const InvScale* sc_up;     // [L]  N^-1 * [(Q_j/q_i)^-1]_{q_i}
    const InvScale* sc_dn;     // [K]  N^-1 * [(P/p_k)^-1]_{p_k}
    const u64* up_hatinv;      // [L][2]  [(Q_j/q_i)^-1]_{q_i} and Shoup companion (stand-alone ModUp)
    const u64* dn_hatinv;      // [K][2]
    const u64* up_chat;        // [L][D]  (Q_j/q_i) * 2^64 mod m_t   (0 inside the digit)
    const double* up_chat_fp;  // [L][D]  (Q_j/q_i) mod m_t as a double (FpAr targets)
    const u32* up_fp_ok;       // [dnum][D] 1 if target t of digit j may convert on the FP64 pipe: target and
                               //           all sources FpAr primes, largest source <= 2 * target
    const u64* dn_chat;        // [K][L]  (P/p_k) * 2^64 mod q_i
    const double* dn_chat_fp;  // [K][L]  (P/p_k) mod q_i as a double (FpAr targets)
    const u32* dn_fp_ok;       // [L]  1 if q_i may convert on the FP64 pipe (FpAr prime, at least 2^28)
    const PinvConst* pinv;     // [L]     P^-1 mod q_i
    const u64* pmod;           // [L]     P mod q_i
    // conversion on the matrix cores (conv_mfma_kernel): target tiles and constant operands per digit; n_tiles = 0
    // when the view does not use it (fewer than 2 or more than 8 sources, or no FpAr target)
    const struct ConvTile* up_tiles;  // [dnum][up_tstride]
    const u64* up_aop;                // [dnum][up_tstride][up_ks][64]
    const struct ConvTile* dn_tiles;  // [dn_ntiles]
    const u64* dn_aop;                // [dn_ntiles][dn_ks][64]
    u32 up_ntiles, up_tstride, up_ks, dn_ntiles, dn_ks;  // tiles in use (most over the digits), tiles stored per digit
    u32 logN, L, K, dnum, alpha, D;
    u32 Lfull;  // q-limbs of the whole prime chain
    u32 Lq;     // limbs 0 .. Lq-1 of this basis are q-limbs of the chain, the rest its special limbs
    // A Tables value describes one level: the basis q_0..q_{L-1}, p_0..p_{K-1} with L <= Lfull active
    // q-limbs, dnum = ceil(L/alpha) digits (the last one possibly partial) and limb indices 0..D-1 over
    // that basis.  The per-prime tables (tw_int, tw_fp, pc, sc_plain) and switching keys are laid out
    // over the whole chain of Lfull + K primes: phys() maps a limb index of the level to them.  All
    // other tables are per level and indexed by the level's limb indices.
    // Three kinds of Tables exist: a level (L active q-limbs, K special limbs, Lq = L); a rescale step
    // (L targets, K = 1 source = q-limb L, Lq = L + 1); a ModDown merged with the rescale after it (L
    // targets, K sources = q-limb L followed by the special limbs, Lq = L + 1).
    __host__ __device__ __forceinline__ u32 phys(u32 i) const { return i < Lq ? i : i + (Lfull - Lq); }
};

// slot j of sigma_g(f) in evaluation form reads slot eval_perm(j) of f
__device__ __forceinline__ u32 eval_perm(u32 j, u32 g, u32 logN) {
    const u32 two_n_mask = (2u << logN) - 1;
    u32 e = (g * (2 * (__brev(j) >> (32 - logN)) + 1)) & two_n_mask;
    return __brev((e - 1) >> 1) >> (32 - logN);
}

// Limb addressing of the plain transform passes: instance `inst`, limb l of n_l:
//   word offset (inst'*gs + first + l) * N, prime index prime_base + l, where inst' = inst unless
//   skip_alpha != 0: then instances enumerate the digits that do NOT own limb first + l
//   (inst' = inst + 1 from the owning digit (first + l) / skip_alpha on).
struct LimbSel {
    u32 n_l, n_inst, gs, first, prime_base, skip_alpha;
};
__device__ __forceinline__ size_t limb_offset(const LimbSel& s, u32 inst, u32 l) {
    if (s.skip_alpha && inst >= (s.first + l) / s.skip_alpha) inst++;
    return (size_t)inst * s.gs + s.first + l;
}

// Layout CP of the 16 words of a lane in a 256-word row (lane e0 of the row's 16): register kk holds word
// (kk/2)*32 + e0*2 + kk%2, i.e. eight adjacent pairs: every global access of the inner product that does not feed a
// transform directly (keys, own-digit operands, results) is a 16-byte access per lane, half the memory
// instructions of the one-word-per-access layout CA.  The per-instruction cost of the address path, not the
// bytes, is what the kernel's memory side was bound by.
typedef u64 u64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32 cp_word(u32 e0, int kk) { return (u32)(kk >> 1) * 32 + e0 * 2 + (u32)(kk & 1); }
template <bool NT>
__device__ __forceinline__ void load_row_cp(const u64* row, u32 e0, u64 (&o)[16]) {
#pragma unroll
    for (int k2 = 0; k2 < 8; k2++) {
        const u64x2* p = reinterpret_cast<const u64x2*>(row + k2 * 32 + e0 * 2);
        const u64x2 t = NT ? __builtin_nontemporal_load(p) : *p;
        o[2 * k2] = t.x, o[2 * k2 + 1] = t.y;
    }
}
template <bool NT = true>
__device__ __forceinline__ void store_row_cp(u64* row, u32 e0, const u64 (&v)[16]) {
#pragma unroll
    for (int k2 = 0; k2 < 8; k2++) {
        u64x2 t;
        t.x = v[2 * k2], t.y = v[2 * k2 + 1];
        u64x2* p = reinterpret_cast<u64x2*>(row + k2 * 32 + e0 * 2);
        if (NT) __builtin_nontemporal_store(t, p);
        else *p = t;
    }
}
// between the contiguous-pass layout CB (word e0*16 + k) and CP, through the row's LDS slice
template <class AR>
__device__ __forceinline__ void exchange_cb_to_cp(typename AR::T (&x)[16], u64* l, u32 e0) {
    row_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) l[pad16(e0 * 16 + k)] = AR::to_raw(x[k]);
    row_sync();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) x[kk] = AR::from_raw(l[pad16(cp_word(e0, kk))]);
}
template <class AR>
__device__ __forceinline__ void exchange_cp_to_cb(typename AR::T (&x)[16], u64* l, u32 e0) {
    row_sync();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) l[pad16(cp_word(e0, kk))] = AR::to_raw(x[kk]);
    row_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = AR::from_raw(l[pad16(e0 * 16 + k)]);
}
// Row `row_off/256` of sigma_g(f) in layout CP.  In evaluation order the automorphism maps a 256-word row onto one
// source row (the row index is the bit-reversed low part of the exponent index, and multiplication by g keeps low
// parts among themselves), so the source row is loaded whole with 16-byte accesses, staged in the row's LDS
// slice and permuted there, instead of one scattered 8-byte global access per word.
__device__ __forceinline__ void gather_row_cp(const u64* limb, u32 row_off, u32 gal, u32 logN, u64* l, u32 e0, u64 (&o)[16]) {
    const u32 src_row = eval_perm(row_off, gal, logN) >> 8;
    load_row_cp<false>(limb + (size_t)src_row * 256, e0, o);
    row_sync();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) l[pad16(cp_word(e0, kk))] = o[kk];
    row_sync();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) o[kk] = l[pad16(eval_perm(row_off + cp_word(e0, kk), gal, logN) & 255)];
}

// most rotations (each with its own key and Galois element) one launch can be given
#define CKKS_ROT_CHUNK 16

// ============================================================ inverse transform, first pass
enum InvLoad { INV_PLAIN = 0, INV_TENSOR = 1, INV_ROT = 2 };
struct InvContigArgs {
    const u64* src;   // PLAIN: canonical eval-form limbs addressed by sel; TENSOR: ct1; ROT: ct
    const u64* src2;  // TENSOR: ct2
    u64* dst;         // raw inverse-lazy words, addressed by dsel
    LimbSel sel, dsel;
    u32 galois[CKKS_ROT_CHUNK];  // ROT: [0], or one per instance when per_inst is set
    u32 per_inst;
};

template <class AR, int A, int LOAD>
__device__ __forceinline__ void inv_contig_body(const InvContigArgs& a, const Tables& tb, u64* lds, u32 l, u32 tile,
                                                u32 inst) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    const u32 pi = tb.phys(a.sel.prime_base + l);
    const PrimeConst pc = tb.pc[pi];
    const typename AR::Mod m = AR::mod(pc);
    const u64* ti = tb.tw_int + (size_t)pi * 4 * N;
    const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
    u64* lrow = lds + ch * 272;
    T x[16];
    // operands arrive in layout CP (16-byte accesses) and are brought into the pass's layout CB by the exchange
    // that the pass needs anyway; a rotation applies its permutation in that exchange
    if (LOAD == INV_PLAIN) {
        u64 w[16];
        load_row_cp<true>(a.src + limb_offset(a.sel, inst, l) * N + (size_t)r * 256, e0, w);
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::round_reduce(AR::from_canon(w[k], m), m);
        exchange_cp_to_cb<AR>(x, lrow, e0);
    } else if (LOAD == INV_TENSOR) {  // d2 = a1 * a2 on limb l of pair `inst`
        const size_t off = (((size_t)inst * 2 + 1) * tb.L + l) * N + (size_t)r * 256;
        u64 w1[16], w2[16];
        load_row_cp<true>(a.src + off, e0, w1);
        load_row_cp<true>(a.src2 + off, e0, w2);
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::round_reduce(AR::mul_canon(w1[k], w2[k], pc, m), m);
        exchange_cp_to_cb<AR>(x, lrow, e0);
    } else {  // sigma_g(a) on limb l of ciphertext `inst`: the source row, whole, permuted on its way through LDS
        const u32 gal = a.galois[a.per_inst ? inst : 0];
        const u64* p = a.src + (((size_t)inst * 2 + 1) * tb.L + l) * N;
        const u32 src_row = eval_perm(r * 256, gal, tb.logN) >> 8;
        u64 w[16];
        load_row_cp<false>(p + (size_t)src_row * 256, e0, w);
        row_sync();
#pragma unroll
        for (int kk = 0; kk < 16; kk++) lrow[pad16(cp_word(e0, kk))] = w[kk];
        row_sync();
#pragma unroll
        for (int k = 0; k < 16; k++)
            x[k] = AR::round_reduce(AR::from_canon(lrow[pad16(eval_perm(r * 256 + e0 * 16 + k, gal, tb.logN) & 255)], m), m);
    }
    NttCore<AR, A>::inv_contig(x, lrow, e0, r, ti, tf, N, m);
    u64* o = a.dst + limb_offset(a.dsel, inst, l) * N + (size_t)r * 256;
#pragma unroll
    for (int k = 0; k < 16; k++) o[k * 16 + e0] = AR::to_raw(AR::round_reduce(x[k], m));
}

// Every transform kernel is compiled once per arithmetic and launched on a run of consecutive
// limbs [run.first, run.first + run.count) whose primes all use that arithmetic.
struct LimbRun {
    u32 first, count;
};

template <class AR, int A, int LOAD>
__global__ __launch_bounds__(256) void inv_contig_kernel(InvContigArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[NTT_LDS_WORDS];
    constexpr u32 TILES = (1u << A) / 16;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.sel.n_inst, run.count * TILES, group, inst)) return;
    inv_contig_body<AR, A, LOAD>(a, tb, lds, run.first + group / TILES, group % TILES, inst);
}

// =========================================================== inverse transform, second pass
enum InvScaleSel { SC_PLAIN = 0, SC_UP = 1, SC_DN = 2 };
struct InvStridedArgs {
    u64* data;  // in place: raw inverse-lazy words in, canonical coefficients (times the scale) out
    LimbSel sel;
    u32 scale;   // InvScaleSel
    u32 out_fmt;  // SrcFormat of the stored words: SRC_F64 applies to limbs of FpAr primes only (others stay canonical)
};

template <class AR, int A>
__device__ __forceinline__ void inv_strided_body(const InvStridedArgs& a, const Tables& tb, u64* lds, u32 l, u32 tile,
                                                 u32 inst) {
    typedef typename AR::T T;
    typedef NttCore<AR, A> C;
    const u32 N = 1u << tb.logN, tid = threadIdx.x;
    const u32 vi = a.sel.prime_base + l, pi = tb.phys(vi);
    const typename AR::Mod m = AR::mod(tb.pc[pi]);
    const u64* ti = tb.tw_int + (size_t)pi * 4 * N;
    const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
    const InvScale sc = a.scale == SC_PLAIN ? tb.sc_plain[pi] : a.scale == SC_UP ? tb.sc_up[vi] : tb.sc_dn[vi - tb.L];
    const u32 c = tid % C::TC, r0 = tid / C::TC, col = tile * C::TC + c;
    u64* base = a.data + limb_offset(a.sel, inst, l) * N;
    T x[16];
    if constexpr (A > 4) {
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::from_raw(base[(size_t)(r0 * 16 + k) * 256 + col]);
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = AR::from_raw(base[(size_t)(k * C::RB + r0) * 256 + col]);
    }
    C::inv_strided_but_last(x, lds, tid, ti, tf, N, m);
#pragma unroll
    for (int k = 0; k < 8; k++) {
        u64 ox, oy;
        AR::bfly_inv_last(x[k], x[k + 8], sc, m, a.out_fmt, ox, oy);
        base[(size_t)(k * C::RB + r0) * 256 + col] = ox;
        base[(size_t)((k + 8) * C::RB + r0) * 256 + col] = oy;
    }
}

#ifndef CKKS_INV_STRIDED_WAVES
#define CKKS_INV_STRIDED_WAVES 6
#endif
template <class AR, int A>
__global__ __launch_bounds__(256, (A == 8 && INV_STRIDED_HALF_EXCHANGE) ? CKKS_INV_STRIDED_WAVES : 4) void inv_strided_kernel(InvStridedArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[(A == 8 && INV_STRIDED_HALF_EXCHANGE) ? 2048 : 4096];
    constexpr u32 TILES = (1u << A) / 16;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.sel.n_inst, run.count * TILES, group, inst)) return;
    inv_strided_body<AR, A>(a, tb, lds, run.first + group / TILES, group % TILES, inst);
}

// ============================================================ forward transform, first pass
struct FwdStridedArgs {
    const u64* src;  // canonical coefficients addressed by sel
    u64* dst;        // raw forward-lazy words, same addressing (in place when dst == src)
    LimbSel sel;
};

// stages + store shared by the plain and the conversion-fused first pass; x in layout SA
template <class AR, int A>
__device__ __forceinline__ void fwd_strided_finish(typename AR::T (&x)[16], const Tables& tb, u64* lds, u32 vi,
                                                   u64* dst, u32 tile) {
    typedef NttCore<AR, A> C;
    const u32 N = 1u << tb.logN, pi = tb.phys(vi);
    const u32 tid = threadIdx.x;
    const typename AR::Mod m = AR::mod(tb.pc[pi]);
    const u64* ti = tb.tw_int + (size_t)pi * 4 * N;
    const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
    const u32 c = tid % C::TC, r0 = tid / C::TC, col = tile * C::TC + c;
    C::fwd_strided(x, lds, tid, ti, tf, N, m);
    if constexpr (A > 4) {
#pragma unroll
        for (int k = 0; k < 16; k++) __builtin_nontemporal_store(AR::to_raw(AR::round_reduce(x[k], m)), &dst[(size_t)(r0 * 16 + k) * 256 + col]);
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++)
            dst[(size_t)(k * C::RB + r0) * 256 + col] = AR::to_raw(AR::round_reduce(x[k], m));
    }
}

template <class AR, int A>
__global__ __launch_bounds__(256) void fwd_strided_kernel(FwdStridedArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[4096];
    typedef NttCore<AR, A> C;
    constexpr u32 TILES = (1u << A) / 16;
    const u32 N = 1u << tb.logN, tid = threadIdx.x;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.sel.n_inst, run.count * TILES, group, inst)) return;
    const u32 l = run.first + group / TILES, tile = group % TILES, pi = a.sel.prime_base + l;
    const size_t off = limb_offset(a.sel, inst, l) * N;
    const typename AR::Mod m = AR::mod(tb.pc[tb.phys(pi)]);
    const u32 c = tid % C::TC, r0 = tid / C::TC, col = tile * C::TC + c;
    typename AR::T x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = AR::from_canon(a.src[off + (size_t)(k * C::RB + r0) * 256 + col], m);
    fwd_strided_finish<AR, A>(x, tb, lds, pi, a.dst + off, tile);
}

// ============================== base conversion fused into the first forward pass of its targets
// CONV_UP: group = (b, digit j, tile); sources y [b][L][N] = coefficients times [(Q_j/q_i)^-1], limbs of
//          FpAr primes stored as doubles; targets = the primes outside digit j; dst dt [b][dnum][D][N].
// CONV_DN: group = (g, tile); sources y = special limbs [g][K][N] (canonical words); targets = q-limbs;
//          dst cv [g][L][N].
// A workgroup converts TB consecutive target primes of the run from one load of the sources (the
// sources come from L2, whose bandwidth is what bounds a one-target-per-workgroup version), then
// runs the first forward pass of each target in turn.
enum ConvDir { CONV_UP = 1, CONV_DN = 2 };
struct ConvArgs {
    const u64* src;
    u64* dst;
    u32 groups_outer;  // CONV_UP: batch; CONV_DN: number of g
    u32 src_fmt;       // SrcFormat of the source words: SRC_DIGITS, or the natural format (the launcher picks the instantiation)
};
// a source word as a canonical integer; DG: the sources are SRC_DIGITS words, else they are in their natural
// format (FpAr-prime sources of ModUp as doubles, everything else canonical)
template <bool DG>
__device__ __forceinline__ u64 conv_src_int(u64 w, bool f64_word) {
    return DG ? digits_decode(w) : f64_word ? f64_to_u64(FpAr::from_raw(w)) : w;
}

template <class AR, int A, int DIR, int TB, bool DG = false>
__global__ __launch_bounds__(256, AR::is_fp ? 3 : 2) void conv_fwd_strided_kernel(ConvArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[4096];
    typedef NttCore<AR, A> C;
    typedef typename AR::T T;
    constexpr u32 TILES = (1u << A) / 16;
    const u32 N = 1u << tb.logN, tid = threadIdx.x;
    const u32 n_inst = (run.count + TB - 1) / TB;
    u32 group, inst, tile, ns, src_prime, chat_stride;
    const u64* src;
    u64* dst0;  // limb 0 of the destination group
    const u64* chat;
    const double* chat_fp;
    const u32* fp_ok;
    u32 own_lo = 0xffffffffu, own_hi = 0xffffffffu;  // target primes in [own_lo, own_hi) are skipped
    if (DIR == CONV_UP) {
        if (!xcd_decode(blockIdx.x, n_inst, a.groups_outer * tb.dnum * TILES, group, inst)) return;
        tile = group % TILES;
        const u32 bj = group / TILES, j = bj % tb.dnum, b = bj / tb.dnum;
        src = a.src + ((size_t)b * tb.L + (size_t)j * tb.alpha) * N;
        dst0 = a.dst + ((size_t)b * tb.dnum + j) * tb.D * N;
        chat = tb.up_chat + (size_t)j * tb.alpha * tb.D;
        chat_fp = tb.up_chat_fp + (size_t)j * tb.alpha * tb.D;
        fp_ok = tb.up_fp_ok + (size_t)j * tb.D;
        // the last digit of a level may hold fewer than alpha limbs
        own_lo = j * tb.alpha, own_hi = (j + 1) * tb.alpha < tb.L ? (j + 1) * tb.alpha : tb.L;
        chat_stride = tb.D, ns = own_hi - own_lo, src_prime = own_lo;
    } else {
        if (!xcd_decode(blockIdx.x, n_inst, a.groups_outer * TILES, group, inst)) return;
        tile = group % TILES;
        const u32 g = group / TILES;
        src = a.src + (size_t)g * tb.K * N;
        dst0 = a.dst + (size_t)g * tb.L * N;
        chat = tb.dn_chat;
        chat_fp = tb.dn_chat_fp;
        fp_ok = tb.dn_fp_ok;
        chat_stride = tb.L, ns = tb.K, src_prime = tb.L;
    }
    u32 pi[TB];
    bool valid[TB], any = false, all_fp = AR::is_fp;
#pragma unroll
    for (int t = 0; t < TB; t++) {
        pi[t] = run.first + inst * TB + t;
        valid[t] = pi[t] < run.first + run.count && !(pi[t] >= own_lo && pi[t] < own_hi);
        if (!valid[t]) pi[t] = run.first;  // any prime of the run: its result is dropped
        any = any || valid[t];
        all_fp = all_fp && (!valid[t] || fp_ok[pi[t]]);
    }
    if (!any) return;
    const u32 c = tid % C::TC, r0 = tid / C::TC, col = tile * C::TC + c;
    const u32 rot = ns ? (inst + tile) % ns : 0;  // workgroups sharing sources walk them in different orders
    T x[TB][16];
    if (all_fp) {
        // FP64 pipe: every product reduced lazily (|.| <= 1.25 q), at most 18 of them accumulated between two
        // reductions of the accumulator (8 sources; ModDown sources count twice).  The 16
        // words of a lane are converted in two halves so that accumulators and staged sources stay small.
        FpAr::Mod fm[TB];
#pragma unroll
        for (int t = 0; t < TB; t++) fm[t] = FpAr::mod(tb.pc[tb.phys(pi[t])]);
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            double acc[TB][8];
#pragma unroll
            for (int t = 0; t < TB; t++)
#pragma unroll
                for (int k = 0; k < 8; k++) acc[t][k] = 0.0;
            // the loads of source i+1 are issued before the arithmetic on source i (software pipeline)
            u64 cur[8], nxt[8];
            {
                const u64* s0 = src + (size_t)rot * N;
#pragma unroll
                for (int k = 0; k < 8; k++) cur[k] = s0[(size_t)((hf * 8 + k) * C::RB + r0) * 256 + col];
            }
            // rounds of 8 sources: with more than 8, the accumulators go back to |acc| <= q/2 between rounds
            for (u32 g0 = 0; g0 < ns; g0 += 8) {
                const u32 ge = g0 + 8 < ns ? g0 + 8 : ns;
                for (u32 i0 = g0; i0 < ge; i0++) {
                    const u32 i = i0 + rot < ns ? i0 + rot : i0 + rot - ns;
                    if (i0 + 1 < ns) {
                        const u32 in = i0 + 1 + rot < ns ? i0 + 1 + rot : i0 + 1 + rot - ns;
                        const u64* sn = src + (size_t)in * N;
#pragma unroll
                        for (int k = 0; k < 8; k++) nxt[k] = sn[(size_t)((hf * 8 + k) * C::RB + r0) * 256 + col];
                    }
                    if (DIR == CONV_UP) {  // sources are doubles holding canonical residues of ~the targets' size
                        double cf[TB];
#pragma unroll
                        for (int t = 0; t < TB; t++) cf[t] = chat_fp[(size_t)i * chat_stride + pi[t]];
#pragma unroll
                        for (int k = 0; k < 8; k++) {
                            const double y = DG ? u64_to_f64(digits_decode(cur[k])) : FpAr::from_raw(cur[k]);
#pragma unroll
                            for (int t = 0; t < TB; t++) acc[t][k] += FpAr::mulmod_lazy(y, cf[t], fm[t]);
                        }
                    } else {  // sources are words below 2^61: brought below the target first, then one product each
                        double cl[TB];
#pragma unroll
                        for (int t = 0; t < TB; t++) cl[t] = chat_fp[(size_t)i * chat_stride + pi[t]];
#pragma unroll
                        for (int k = 0; k < 8; k++) {
                            const u64 y = DG ? digits_decode(cur[k]) : cur[k];
                            const double ya = (double)(u32)(y >> 30) * 1073741824.0, yl = (double)(u32)(y & 0x3fffffffu);
#pragma unroll
                            for (int t = 0; t < TB; t++)
                                acc[t][k] += FpAr::mulmod_lazy(FpAr::reduce_split(ya, yl, fm[t]), cl[t], fm[t]);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 8; k++) cur[k] = nxt[k];
                }
                if (ge < ns) {
#pragma unroll
                    for (int t = 0; t < TB; t++)
#pragma unroll
                        for (int k = 0; k < 8; k++) acc[t][k] = FpAr::reduce(acc[t][k], fm[t]);
                }
            }
#pragma unroll
            for (int t = 0; t < TB; t++) {
                const typename AR::Mod m = AR::mod(tb.pc[tb.phys(pi[t])]);
#pragma unroll
                for (int k = 0; k < 8; k++) x[t][hf * 8 + k] = AR::from_f64_lazy(acc[t][k], m);
            }
        }
    } else if (!AR::is_fp) {
        // integer pipe: 128-bit accumulation against Montgomery-form constants, one reduction per target;
        // in two halves of eight words like the FP64 path
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            u128w acc[TB][8];
#pragma unroll
            for (int t = 0; t < TB; t++)
#pragma unroll
                for (int k = 0; k < 8; k++) acc[t][k] = u128w{0, 0};
            // 8 terms (each below 2^61 * q) stay below q * 2^64, the bound of the reduction: with more sources,
            // q * 2^64 is taken off after every round of 8 terms
            for (u32 g0 = 0; g0 < ns; g0 += 8) {
                const u32 ge = g0 + 8 < ns ? g0 + 8 : ns;
                for (u32 i0 = g0; i0 < ge; i0++) {
                    const u32 i = i0 + rot < ns ? i0 + rot : i0 + rot - ns;
                    const u64* si = src + (size_t)i * N;
                    const bool src_fp = DIR == CONV_UP && tb.pc[tb.phys(src_prime + i)].fp;
                    u64 cc[TB];
#pragma unroll
                    for (int t = 0; t < TB; t++) cc[t] = chat[(size_t)i * chat_stride + pi[t]];
#pragma unroll
                    for (int k = 0; k < 8; k++) {
                        const u64 y = conv_src_int<DG>(si[(size_t)((hf * 8 + k) * C::RB + r0) * 256 + col], src_fp);
#pragma unroll
                        for (int t = 0; t < TB; t++) mac128(acc[t][k], y, cc[t]);
                    }
                }
                if (ns > 8) {
#pragma unroll
                    for (int t = 0; t < TB; t++) {
                        const u64 qt = tb.pc[tb.phys(pi[t])].q;
#pragma unroll
                        for (int k = 0; k < 8; k++) acc[t][k].hi = csub(acc[t][k].hi, qt);
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < TB; t++) {
                const PrimeConst pc = tb.pc[tb.phys(pi[t])];
                const typename AR::Mod m = AR::mod(pc);
#pragma unroll
                for (int k = 0; k < 8; k++) x[t][hf * 8 + k] = AR::from_canon(redc(acc[t][k], pc.q, pc.qneg), m);
            }
        }
    } else {
        // FpAr targets whose sources do not fit the FP64 bounds: integer conversion, one target at a time
        for (int t = 0; t < TB; t++) {
            const PrimeConst pc = tb.pc[tb.phys(pi[t])];
            const typename AR::Mod m = AR::mod(pc);
            u128w acc[16];
#pragma unroll
            for (int k = 0; k < 16; k++) acc[k] = u128w{0, 0};
            for (u32 i = 0; i < ns; i++) {
                const u64* si = src + (size_t)i * N;
                const bool src_fp = DIR == CONV_UP && tb.pc[tb.phys(src_prime + i)].fp;
                const u64 cc = chat[(size_t)i * chat_stride + pi[t]];
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    const u64 y = conv_src_int<DG>(si[(size_t)(k * C::RB + r0) * 256 + col], src_fp);
                    mac128(acc[k], y, cc);
                }
                if (ns > 8 && ((i & 7) == 7 || i + 1 == ns)) {
#pragma unroll
                    for (int k = 0; k < 16; k++) acc[k].hi = csub(acc[k].hi, pc.q);
                }
            }
#pragma unroll
            for (int tt = 0; tt < TB; tt++)
                if (tt == t) {
#pragma unroll
                    for (int k = 0; k < 16; k++) x[tt][k] = AR::from_canon(redc(acc[k], pc.q, pc.qneg), m);
                }
        }
    }
#pragma unroll
    for (int t = 0; t < TB; t++) {
        if (t) __syncthreads();  // the previous target's exchange must have been read
        if (valid[t]) fwd_strided_finish<AR, A>(x[t], tb, lds, pi[t], dst0 + (size_t)pi[t] * N, tile);
        else if (A > 4) __syncthreads();  // keep barrier counts equal (fwd_strided holds one barrier)
    }
}


// ===================== base conversion on the matrix cores, fused into the first forward pass of FpAr targets
// out_t = sum_i y_i * chat_{i,t} mod m_t as an 8-bit integer matrix product.  Every source word arrives as eight
// signed base-256 digits (SRC_DIGITS), y_i = sum_b d_{i,b} 256^b; the digit weight is folded into the constant,
// C_{(i,b),t} = centred (chat_{i,t} * 256^b mod m_t), itself cut into seven signed digits C = sum_g c_g 256^g.  Then
//   S_{t,g}[n] = sum_{(i,b)} c_g(C_{(i,b),t}) * d_{i,b}(y_i[n])          (v_mfma_i32_32x32x32_i8, |S| < 2^21)
//   out_t[n]  == sum_g 256^g S_{t,g}[n]  (mod m_t),
// recombined exactly in FP64 (conv_recombine).  One 32x32x32 product handles 32 coefficients (columns) and 32
// rows = up to 4 targets x 8 digit rows, over 32 values of (i,b) = four sources (lane half h holds the digit words
// of sources 4*ks + 2*h and 4*ks + 2*h + 1 in its 16 operand bytes, the constant operand the matching bytes);
// ceil(ns/4) products accumulate all sources.  Row m of the constant tile sits in accumulator a = (m/8)*4 + m%4 of lane half (m/4)%2, so a lane
// holds all digits of its targets: target slot tl = h * ntt + a/8, digit a%8 (ntt = targets per lane, 1 or 2).
//
// A lane converts, for s = 0, 1 and every k < 16, coefficient (row k*RB + r0, column c) of the tile, with
// (r0, c) from pp = wave*64 + s*32 + lane%32 exactly as tid maps to (r0, c) in layout SA: the 16 values k of one
// (s, target) are the inputs of the first four forward stages, which therefore run in the lane that converted
// them; the exchange for the remaining stages goes through LDS target by target.
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));
struct ConvTile {
    u32 target[4];  // limb index of target slot tl within the destination group; 0xffffffff = unused slot
    u32 ntt;        // targets per lane half (1 or 2); 0 = unused tile
    u32 pad[3];
};
struct MfmaConvArgs {
    const u64* src;         // SRC_DIGITS words: CONV_UP [b][L][N], CONV_DN [g][K][N]
    u64* dst;               // raw forward-lazy words after the first pass: CONV_UP dt [b][dnum][D][N], CONV_DN cv [g][L][N]
    const ConvTile* tiles;  // [digits][n_tiles]
    const u64* aop;         // [digits][n_tiles][KS][64][2] constant operands, one 16-byte row fragment per lane
    u32 groups_outer;       // CONV_UP: batch; CONV_DN: number of g
    u32 n_tiles;            // tiles launched per digit
    u32 tile_stride;        // tiles stored per digit
};

// sum_g 256^g S_g reduced to |.| <= (0.5 + 2^-15) m, exactly: lo = digits 0..3 (below 2^46), hi = digits 4..6 times
// 2^32 (an integer multiple of 2^32 with 38 significant bits: exact); the quotient estimate of (hi + lo) / m is off
// by less than 2^-15 before rounding, hi - c*m is an integer below 2^53 in magnitude, so the fma and the sum are exact.
// (Summing the digits with 64-bit integer multiply-adds onto the bit pattern of a double, which avoids the
// i32 -> f64 conversions, was measured 5 % slower on the kernel.)
__device__ __forceinline__ double conv_recombine(const v16i& s, int b, const FpAr::Mod& m) {
    const double lo = __builtin_fma((double)s[b + 3], 16777216.0,
                                    __builtin_fma((double)s[b + 2], 65536.0, __builtin_fma((double)s[b + 1], 256.0, (double)s[b])));
    const double hi = __builtin_fma((double)s[b + 6], 281474976710656.0,
                                    __builtin_fma((double)s[b + 5], 1099511627776.0, (double)s[b + 4] * 4294967296.0));
    const double c = __builtin_rint((hi + lo) * m.qinv);
    return __builtin_fma(-c, m.q, hi) + lo;
}

template <int A, int KS, int DIR, int NTT>
__global__ __launch_bounds__(256, NTT == 1 ? 3 : 2) void conv_mfma_kernel(MfmaConvArgs a, Tables tb) {
    __shared__ u64 lds[4096];
    typedef NttCore<FpAr, A> C;
    constexpr u32 TILES = (1u << A) / 16;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, h = lane >> 5;
    const u32 n_dig = DIR == CONV_UP ? tb.dnum : 1;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.n_tiles, a.groups_outer * n_dig * TILES, group, inst)) return;
    const u32 tile = group % TILES;
    u32 j = 0, ns;
    const u64* src;
    u64* dst0;
    if (DIR == CONV_UP) {
        const u32 bj = group / TILES, b = bj / tb.dnum;
        j = bj % tb.dnum;
        const u32 own_lo = j * tb.alpha, own_hi = (j + 1) * tb.alpha < tb.L ? (j + 1) * tb.alpha : tb.L;
        ns = own_hi - own_lo;
        src = a.src + ((size_t)b * tb.L + own_lo) * N;
        dst0 = a.dst + ((size_t)b * tb.dnum + j) * tb.D * N;
    } else {
        const u32 g = group / TILES;
        ns = tb.K;
        src = a.src + (size_t)g * tb.K * N;
        dst0 = a.dst + (size_t)g * tb.L * N;
    }
    const ConvTile ct = a.tiles[j * a.tile_stride + inst];
    if (ct.ntt == 0) return;  // digits with fewer targets leave their last tiles unused (uniform per workgroup)
    auto slot_target = [&](u32 tl) { return tl == 0 ? ct.target[0] : tl == 1 ? ct.target[1] : tl == 2 ? ct.target[2] : ct.target[3]; };
    v4i aop[KS];
    {
        const v4i* ap = reinterpret_cast<const v4i*>(a.aop) + (size_t)(j * a.tile_stride + inst) * KS * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) aop[ks] = ap[ks * 64];
    }
    // this lane's targets: slots h * ntt + tt
    u32 vi[NTT];
    FpAr::Mod fm[NTT];
#pragma unroll
    for (int tt = 0; tt < NTT; tt++) {
        vi[tt] = (u32)tt < ct.ntt ? slot_target(h * ct.ntt + tt) : 0xffffffffu;
        fm[tt] = FpAr::mod(tb.pc[tb.phys(vi[tt] != 0xffffffffu ? vi[tt] : 0)]);
    }
    double x[2][NTT][16];
    // 32 coefficient groups g = s*16 + k per lane.  The source words of group g + PF are requested before the products
    // of group g are issued; scheduling barriers keep the compiler from hoisting every load of the unrolled loop
    // (which would spill).
    constexpr int PF = 2;  // deeper prefetch (4, 6, 8 groups) changes nothing: the words come from L2
    // this lane half supplies the digits of sources 4*ks + 2*h and the next one; beyond the last source any valid word
    // will do (the constant rows of those sources are zero)
    const u64* sp[2 * KS];
#pragma unroll
    for (int q = 0; q < 2 * KS; q++) {
        const u32 i = 4 * (q >> 1) + 2 * h + (q & 1);
        sp[q] = src + (size_t)(i < ns ? i : ns - 1) * N + tile * C::TC;
    }
    auto src_off = [&](int g) {
        const u32 pp = wave * 64 + (g >> 4) * 32 + n;
        return (u32)(((g & 15) * C::RB + pp / C::TC) * 256 + pp % C::TC);
    };
    u64 bw[PF + 1][2 * KS];
#pragma unroll
    for (int g = 0; g < PF; g++) {
#pragma unroll
        for (int q = 0; q < 2 * KS; q++) bw[g][q] = sp[q][src_off(g)];
    }
#pragma unroll
    for (int g = 0; g < 32; g++) {
        if (g + PF < 32) {
#pragma unroll
            for (int q = 0; q < 2 * KS; q++) bw[(g + PF) % (PF + 1)][q] = sp[q][src_off(g + PF)];
        }
        v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            const u64 w0 = bw[g % (PF + 1)][2 * ks], w1 = bw[g % (PF + 1)][2 * ks + 1];
            const v4i bop = {(int)(u32)w0, (int)(u32)(w0 >> 32), (int)(u32)w1, (int)(u32)(w1 >> 32)};
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(aop[ks], bop, acc, 0, 0, 0);
        }
#pragma unroll
        for (int tt = 0; tt < NTT; tt++) x[g >> 4][tt][g & 15] = conv_recombine(acc, tt * 8, fm[tt]);
        __builtin_amdgcn_sched_barrier(0);
    }
    // first four forward stages of every (s, target) set, in place (|x| <= 0.51 q on entry, below 7 q after)
#pragma unroll
    for (int tt = 0; tt < NTT; tt++) {
        if (vi[tt] == 0xffffffffu) continue;
        const double* tf = tb.tw_fp + (size_t)tb.phys(vi[tt]) * 2 * N;
#pragma unroll
        for (int st = 0; st < 4; st++) {
            const int d = 8 >> st;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                if (k & d) continue;
                const FpAr::Tw w = FpAr::tw(nullptr, tf, (1u << st) + (k >> (4 - st)), N, false);
#pragma unroll
                for (int s = 0; s < 2; s++) FpAr::bfly_fwd<false>(x[s][tt][k], x[s][tt][k + d], w, fm[tt]);
            }
        }
    }
    // remaining stages and store, one target at a time
#pragma unroll
    for (int tt = 0; tt < NTT; tt++) {
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
            if ((u32)tt >= ct.ntt) continue;
            const u32 t_vi = slot_target(hh * ct.ntt + tt);  // uniform over the workgroup
            if (t_vi == 0xffffffffu) continue;
            const u32 pi = tb.phys(t_vi);
            const FpAr::Mod m = FpAr::mod(tb.pc[pi]);
            u64* dst = dst0 + (size_t)t_vi * N;
            if constexpr (A > 4) {
                __syncthreads();  // the previous target's exchange has been read
                if (h == (u32)hh) {
#pragma unroll
                    for (int s = 0; s < 2; s++) {
                        const u32 pp = wave * 64 + s * 32 + n;
#pragma unroll
                        for (int k = 0; k < 16; k++) lds[k * 256 + pp] = FpAr::to_raw(FpAr::reduce(x[s][tt][k], m));
                    }
                }
                __syncthreads();
                const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
                const u32 c = tid % C::TC, r1 = tid / C::TC, col = tile * C::TC + c;
                double y[16];
#pragma unroll
                for (int k = 0; k < 16; k++) y[k] = FpAr::from_raw(lds[(r1 * 16 + k) * C::TC + c]);
#pragma unroll
                for (int st = 4; st < A; st++) {
                    const int d = 1 << (A - st - 1);
#pragma unroll
                    for (int k = 0; k < 16; k++) {
                        if (k & d) continue;
                        FpAr::bfly_fwd<false>(y[k], y[k + d], FpAr::tw(nullptr, tf, (1u << st) + ((r1 * 16 + k) >> (A - st)), N, false), m);
                    }
                }
#pragma unroll
                for (int k = 0; k < 16; k++)
                    __builtin_nontemporal_store(FpAr::to_raw(FpAr::reduce(y[k], m)), &dst[(size_t)(r1 * 16 + k) * 256 + col]);
            } else {
                if (h == (u32)hh) {
#pragma unroll
                    for (int s = 0; s < 2; s++) {
                        const u32 pp = wave * 64 + s * 32 + n, c = pp % C::TC, r0 = pp / C::TC, col = tile * C::TC + c;
#pragma unroll
                        for (int k = 0; k < 16; k++)
                            dst[(size_t)(k * C::RB + r0) * 256 + col] = FpAr::to_raw(FpAr::reduce(x[s][tt][k], m));
                    }
                }
            }
        }
    }
}

// =========================================================== forward transform, second pass
struct FwdContigArgs {
    u64* data;  // in place: raw forward-lazy words in, canonical evaluation form out
    LimbSel sel;
};

template <class AR, int A>
__device__ __forceinline__ void fwd_contig_body(const FwdContigArgs& a, const Tables& tb, u64* lds, u32 l, u32 tile,
                                                u32 inst) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    const u32 pi = tb.phys(a.sel.prime_base + l);
    const typename AR::Mod m = AR::mod(tb.pc[pi]);
    const u64* ti = tb.tw_int + (size_t)pi * 4 * N;
    const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
    u64* lrow = lds + ch * 272;
    u64* p = a.data + limb_offset(a.sel, inst, l) * N + (size_t)r * 256;
    T x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = AR::from_raw(p[k * 16 + e0]);
    NttCore<AR, A>::fwd_contig(x, lrow, e0, r, ti, tf, N, m);
    row_sync();
#pragma unroll
    for (int k = 0; k < 16; k++) lrow[pad16(e0 * 16 + k)] = AR::canon_fwd(x[k], m);
    row_sync();
    u64 res[16];  // stored in layout CP: 16 bytes per access; cacheable, the caller's next call reads it
#pragma unroll
    for (int kk = 0; kk < 16; kk++) res[kk] = lrow[pad16(cp_word(e0, kk))];
    store_row_cp<false>(p, e0, res);
}

template <class AR, int A>
__global__ __launch_bounds__(256) void fwd_contig_kernel(FwdContigArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[NTT_LDS_WORDS];
    constexpr u32 TILES = (1u << A) / 16;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.sel.n_inst, run.count * TILES, group, inst)) return;
    fwd_contig_body<AR, A>(a, tb, lds, run.first + group / TILES, group % TILES, inst);
}

// ==================================================================== key inner product
// Work item = (limb i of D, tile, instance).  For every digit j the evaluation-form value of the
// extended digit on limb i is produced in registers -- the second forward pass of dt[.][j][i]
// (NTT_INSIDE), or a gather from the already transformed digits (hoisted rotations), or, on the
// digit's own limbs, the switched polynomial itself (copy | a1*a2 | sigma_g(a)) -- multiplied by
// the two key components and accumulated.  q-limbs: c' is stored canonical.  Special limbs: the
// first inverse pass of ModDown runs on the accumulators and raw words are stored.
enum OwnLoad { OWN_COPY = 0, OWN_TENSOR = 1, OWN_ROT = 2 };
struct InnerArgs {
    const u64* dt;    // [inst or 1][dnum][D][N]: raw forward-lazy (NTT_INSIDE) or canonical eval (hoisted)
    const u64* own;   // COPY: d [inst][L][N]; TENSOR: ct1; ROT: ct ([inst][2][L][N]); hoisted: ct [2][L][N]
    const u64* own2;  // TENSOR: ct2
    const u64* key[CKKS_ROT_CHUNK];  // one shared key (index 0) or one per instance (hoisted)
    u32 galois[CKKS_ROT_CHUNK];      // ROT: [0]; hoisted: per instance
    u64* cq;                         // [inst][2][L][N] canonical
    u64* cp;                         // [inst][2][D - split][N] raw inverse-lazy after the first inverse pass
    u32 n_inst;
    u32 split;    // limbs below split are stored to cq ([inst][2][split][N]), the others continue to cp: the number
                  // of q-limbs, or one less when the ModDown that follows also divides by the last q-limb
    u32 per_inst;    // not hoisted: every instance has its own key and Galois element (at most CKKS_ROT_CHUNK instances)
    // FUSED (limbs below split only, launched after the ModDown conversion): the kernel also ends the ModDown
    const u64* cv;              // [inst][2][split][N] converted special part, first forward pass done
    u64* out;                   // [inst][2][split][N]
    const PinvConst* fin_pinv;  // [split] inverse of the product of the ModDown's source primes
};

// Twiddles of one row's second forward pass, kept in LDS for kernels that run that pass several times on the same
// row of the same limb (the inner product: once per digit and twice more when it ends the ModDown).  FP64 limbs
// only: 255 doubles per row.  Words [0, 15): stages 0-3, whose 2^u twiddles are the same for the row's 16 lanes
// (stage u from offset 2^u - 1); then 15 words per lane: stages 4-7, 2^(u-4) twiddles each.  The lane blocks are
// 15 words apart, so the 16 lanes of a row read 16 different bank pairs.  Loaded from the tables once per
// workgroup: the 30 global loads per lane and pass were 14 % of the fused kernel's time.
#define CKKS_ROW_TW_WORDS 256
template <int A>
__device__ __forceinline__ void fill_row_tw(u64* blk, u32 e0, u32 r, const double* tf) {
    if (e0 < 15) {
        const u32 u = 31 - __clz(e0 + 1), off = e0 + 1 - (1u << u);
        blk[e0] = __builtin_bit_cast(u64, tf[(1u << (A + u)) + (r << u) + off]);
    }
#pragma unroll
    for (int u = 4; u < 8; u++) {
#pragma unroll
        for (int t = 0; t < (1 << (u - 4)); t++)
            blk[15 + e0 * 15 + (1 << (u - 4)) - 1 + t] = __builtin_bit_cast(u64, tf[(1u << (A + u)) + (r << u) + (e0 << (u - 4)) + t]);
    }
    row_sync();
}
struct RowTwLds {
    const u64* blk;
    u32 e0;
    __device__ __forceinline__ FpAr::Tw get(int u, u32 w) const {
        const u32 t = w >> (8 - u);
        const u32 at = u < 4 ? (1u << u) - 1 + t : 15 + e0 * 15 + (1u << (u - 4)) - 1 + (t - (e0 << (u - 4)));
        return FpAr::Tw{__builtin_bit_cast(double, blk[at])};
    }
};

template <class AR, int A, int OWN, bool HOISTED, bool FUSED>
__device__ __forceinline__ void ks_inner_body(const InnerArgs& a, const Tables& tb, u64* lds, u32 i, u32 tile,
                                              u32 inst) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    const u32 L = tb.L, D = tb.D;
    const u32 pi = tb.phys(i), Dkey = tb.Lfull + tb.K;  // keys are laid out over the whole chain
    const PrimeConst pc = tb.pc[pi];
    const typename AR::Mod m = AR::mod(pc);
    const u64* ti = tb.tw_int + (size_t)pi * 4 * N;
    const double* tf = tb.tw_fp + (size_t)pi * 2 * N;
    u64* lrow = lds + ch * 272;
    const u32 row_off = r * 256;
    const u32 kidx = (HOISTED || a.per_inst) ? inst : 0;
    const u64* key = a.key[kidx] + (size_t)pi * N + row_off;
    const u32 gal = a.galois[kidx];
    const u32 own_digit = i < L ? i / tb.alpha : 0xffffffffu;
    constexpr bool TWL = AR::is_fp && !HOISTED;  // the row's forward twiddles live in LDS
    u64* twblk = lds + NTT_LDS_WORDS + ch * CKKS_ROW_TW_WORDS;
    if constexpr (TWL) fill_row_tw<A>(twblk, e0, r, tf);
    T acc0[16], acc1[16];  // layout CP
#pragma unroll
    for (int k = 0; k < 16; k++) acc0[k] = AR::acc_zero(), acc1[k] = AR::acc_zero();
    for (u32 j = 0; j < tb.dnum; j++) {
        const u64* k0 = key + ((size_t)j * 2 + 0) * Dkey * N;
        const u64* k1 = key + ((size_t)j * 2 + 1) * Dkey * N;
        u64 kv0[16], kv1[16];
        // FpAr issues key loads before the transform so that they are in flight meanwhile: both components
        // where the registers allow it (measured per variant), else the first one only; IntAr has no
        // registers to spare and loads the key at its use
        constexpr bool EARLY0 = AR::is_fp, EARLY1 = AR::is_fp && OWN == OWN_TENSOR;
        if constexpr (EARLY0) load_row_cp<false>(k0, e0, kv0);
        if constexpr (EARLY1) load_row_cp<false>(k1, e0, kv1);
        T v[16];  // the digit on this limb, evaluation form, layout CP
        if (j == own_digit) {
            if (HOISTED) {
                u64 w[16];
                gather_row_cp(a.own + ((size_t)L + i) * N, row_off, gal, tb.logN, lrow, e0, w);
#pragma unroll
                for (int k = 0; k < 16; k++) v[k] = AR::round_reduce(AR::from_canon(w[k], m), m);
            } else if (OWN == OWN_COPY) {
                u64 w[16];
                load_row_cp<false>(a.own + ((size_t)inst * L + i) * N + row_off, e0, w);
#pragma unroll
                for (int k = 0; k < 16; k++) v[k] = AR::round_reduce(AR::from_canon(w[k], m), m);
            } else if (OWN == OWN_TENSOR) {
                // the tensor terms d0 = b1*b2 and d1 = a1*b2 + a2*b1 join c' here as P * d, where a1 and a2 are
                // loaded anyway: (c' + P*d - conv) * P^-1 = (c' - conv) * P^-1 + d, so the kernel that ends the
                // ModDown adds nothing, also when it divides by the last q-limb as well.  One more product
                // between folds: at most 9 * 0.69 q < 2^53, still exact.
                const size_t off = (((size_t)inst * 2 + 1) * L + i) * N + row_off, offb = off - (size_t)L * N;
                const u64 pmod = tb.pmod[i];
#pragma unroll
                for (int k2 = 0; k2 < 8; k2++) {
                    const u32 w = k2 * 32 + e0 * 2;
                    const u64x2 a1 = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(a.own + off + w));
                    const u64x2 a2 = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(a.own2 + off + w));
                    const u64x2 b1 = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(a.own + offb + w));
                    const u64x2 b2 = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(a.own2 + offb + w));
#pragma unroll
                    for (int b = 0; b < 2; b++) {
                        const int k = 2 * k2 + b;
                        v[k] = AR::round_reduce(AR::mul_canon(a1[b], a2[b], pc, m), m);
                        AR::acc_mac(acc0[k], AR::mul_canon(b1[b], b2[b], pc, m), pmod, m);
                        AR::acc_mac(acc1[k], AR::mul_canon(a1[b], b2[b], pc, m) + AR::mul_canon(a2[b], b1[b], pc, m), pmod, m);
                    }
                }
            } else {
                u64 w[16];
                gather_row_cp(a.own + (((size_t)inst * 2 + 1) * L + i) * N, row_off, gal, tb.logN, lrow, e0, w);
#pragma unroll
                for (int k = 0; k < 16; k++) v[k] = AR::round_reduce(AR::from_canon(w[k], m), m);
            }
        } else if (HOISTED) {
            u64 w[16];
            gather_row_cp(a.dt + ((size_t)j * D + i) * N, row_off, gal, tb.logN, lrow, e0, w);
#pragma unroll
            for (int k = 0; k < 16; k++) v[k] = AR::round_reduce(AR::from_canon(w[k], m), m);
        } else {
            const u64* p = a.dt + (((size_t)inst * tb.dnum + j) * D + i) * N + row_off;
#pragma unroll
            for (int k = 0; k < 16; k++) v[k] = AR::from_raw(__builtin_nontemporal_load(&p[k * 16 + e0]));
            if constexpr (TWL) NttCore<AR, A>::fwd_contig_with(v, lrow, e0, RowTwLds{twblk, e0}, m);
            else NttCore<AR, A>::fwd_contig(v, lrow, e0, r, ti, tf, N, m);
#pragma unroll
            for (int k = 0; k < 16; k++) v[k] = AR::round_reduce(v[k], m);
            exchange_cb_to_cp<AR>(v, lrow, e0);
        }
        if constexpr (!EARLY0) load_row_cp<false>(k0, e0, kv0);
#pragma unroll
        for (int k = 0; k < 16; k++) AR::acc_mac(acc0[k], v[k], kv0[k], m);
        if constexpr (!EARLY1) load_row_cp<false>(k1, e0, kv1);
#pragma unroll
        for (int k = 0; k < 16; k++) AR::acc_mac(acc1[k], v[k], kv1[k], m);
        if ((j & 7) == 7) {  // FpAr sums at most 8 lazily reduced products (0.69 q each) between reductions
#pragma unroll
            for (int k = 0; k < 16; k++) acc0[k] = AR::acc_fold(acc0[k], m), acc1[k] = AR::acc_fold(acc1[k], m);
        }
    }
    if (FUSED) {
        // c' stays in registers: out = (c' - second forward pass of the converted special part) * P^-1
        // (+ sigma_g(b) on the first component of a rotation; adding it as P * sigma_g(b) where sigma_g(a) is
        // gathered measured slower: the accumulation loop has no registers for it).  FP64 magnitudes in units
        // of q: c' <= 0.5, v <= 5.2, the product with P^-1 <= 2.9; canonicalised before the store.
        // Opaque copies of the lane coordinates: every address of this part is derived from them, so none of
        // it is computed before the accumulation loop, which has no registers to spare.
        u32 e0f = e0, chf = ch, gal_fin = gal;
        asm volatile("" : "+v"(e0f), "+v"(chf), "+s"(gal_fin));
        const u32 rf = tile * 16 + chf, row_off_f = rf * 256;
        u64* lrow_f = lds + chf * 272;
        const PinvConst pinv = a.fin_pinv[i];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            T v[16];
            const u64* p = a.cv + (((size_t)inst * 2 + t) * a.split + i) * N + row_off_f;
#pragma unroll
            for (int k = 0; k < 16; k++) v[k] = AR::from_raw(__builtin_nontemporal_load(&p[k * 16 + e0f]));
            if constexpr (TWL) NttCore<AR, A>::fwd_contig_with(v, lrow_f, e0f, RowTwLds{lds + NTT_LDS_WORDS + chf * CKKS_ROW_TW_WORDS, e0f}, m);
            else NttCore<AR, A>::fwd_contig(v, lrow_f, e0f, rf, ti, tf, N, m);
            exchange_cb_to_cp<AR>(v, lrow_f, e0f);
            u64 res[16];
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const T fin = AR::acc_finish(t ? acc1[k] : acc0[k], m);
                if constexpr (AR::is_fp) res[k] = AR::to_raw(FpAr::mulmod_lazy(fin - v[k], pinv.d, FpAr::mod(pc)));
                else res[k] = mul_shoup(submod(AR::acc_canon(fin, m), AR::canon_fwd(v[k], m), pc.q), pinv.w, pinv.wp, pc.q);
            }
            if (OWN == OWN_ROT && t == 0) {
                u64 bw[16];
                gather_row_cp(a.own + ((size_t)inst * 2 * L + i) * N, row_off_f, gal_fin, tb.logN, lrow_f, e0f, bw);
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    if constexpr (AR::is_fp) res[k] = AR::to_raw(AR::from_raw(res[k]) + u64_to_f64(bw[k]));
                    else res[k] = addmod(res[k], bw[k], pc.q);
                }
            }
            if constexpr (AR::is_fp) {
#pragma unroll
                for (int k = 0; k < 16; k++) res[k] = FpAr::canon(AR::from_raw(res[k]), FpAr::mod(pc));
            }
            store_row_cp(a.out + (((size_t)inst * 2 + t) * a.split + i) * N + row_off_f, e0f, res);
        }
    } else if (i < a.split) {
        u64 res[16];
#pragma unroll
        for (int t = 0; t < 2; t++) {
#pragma unroll
            for (int k = 0; k < 16; k++) res[k] = AR::acc_canon(AR::acc_finish(t ? acc1[k] : acc0[k], m), m);
            store_row_cp(a.cq + (((size_t)inst * 2 + t) * a.split + i) * N + row_off, e0, res);
        }
    } else {
#pragma unroll
        for (int t = 0; t < 2; t++) {
            T x[16];
#pragma unroll
            for (int k = 0; k < 16; k++) x[k] = AR::acc_finish(t ? acc1[k] : acc0[k], m);
            exchange_cp_to_cb<AR>(x, lrow, e0);
            NttCore<AR, A>::inv_contig(x, lrow, e0, r, ti, tf, N, m);
            u64* o = a.cp + (((size_t)inst * 2 + t) * (D - a.split) + (i - a.split)) * N + row_off;
#pragma unroll
            for (int k = 0; k < 16; k++) o[k * 16 + e0] = AR::to_raw(AR::round_reduce(x[k], m));
        }
    }
}

template <class AR, int A, int OWN, bool HOISTED, bool FUSED>
__global__ __launch_bounds__(256, 2) void ks_inner_kernel(InnerArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[NTT_LDS_WORDS + (AR::is_fp && !HOISTED ? 16 * CKKS_ROW_TW_WORDS : 0)];
    constexpr u32 TILES = (1u << A) / 16;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.n_inst, run.count * TILES, group, inst)) return;
    ks_inner_body<AR, A, OWN, HOISTED, FUSED>(a, tb, lds, run.first + group / TILES, group % TILES, inst);
}

// ===================================================== double-hoisted rotate-multiply-accumulate
// Over the rotations r of the launch and the digits j, on every limb i of the extended basis:
//   C_t[i] += (pt_r[i] * sigma_{g_r}(Dh_j)[i]) * rk_r[j][t][i],   t = 0, 1,
// with Dh_j read by gather from the transformed digits (the polynomial's own limb on the digit that
// owns limb i).  On q-limbs the term pt_r * sigma_{g_r}(b) * P is added to C_0: ModDown divides it by
// P exactly, which gives the same words as adding pt_r * sigma_{g_r}(b) after ModDown.
// C_t is stored canonical, evaluation form: q-limbs in cq, special limbs in cp (ModDown follows).
#define CKKS_DH_CHUNK 32
struct DhInnerArgs {
    const u64* dt;   // [dnum][D][N] canonical evaluation form
    const u64* ct;   // [2][L][N]
    const u64* pt;   // [n_rot][D][N] canonical evaluation form, extended basis; null = the constant 1
    const u64* key[CKKS_DH_CHUNK];
    u32 galois[CKKS_DH_CHUNK];
    u64* cq;         // [2][L][N]
    u64* cp;         // [2][K][N]  (evaluation form here; the inverse transform is a separate launch)
    u32 n_rot;
    u32 accumulate;  // add to what cq / cp already hold (a call with more rotations than one launch takes)
    u32 split;       // limbs below split go to cq ([2][split][N]), the others to cp ([2][D - split][N])
};

// No transform is involved, so the work is element-parallel with few registers per lane (many waves in
// flight hide the gather and key-load latency): work item = (limb i, 256 * EPT consecutive slots), lane
// `tid` owns slots base + k * 256 + tid.
template <class AR, int EPT>
__global__ __launch_bounds__(256) void dh_accum_kernel(DhInnerArgs a, Tables tb, LimbRun run) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, L = tb.L, D = tb.D;
    const u32 chunks = N / (256 * EPT);
    const u32 i = run.first + blockIdx.x / chunks, base = (blockIdx.x % chunks) * (256 * EPT) + tid;
    if (i >= run.first + run.count) return;
    const u32 Dkey = tb.Lfull + tb.K, pi = tb.phys(i);
    const bool is_q = i < L;
    const PrimeConst pc = tb.pc[pi];
    const typename AR::Mod m = AR::mod(pc);
    const u32 own_digit = is_q ? i / tb.alpha : 0xffffffffu;
    const u64 pmod = is_q ? tb.pmod[i] : 0;
    const u64* bp = a.ct + (size_t)(is_q ? i : 0) * N;
    T acc0[EPT], acc1[EPT];
#pragma unroll
    for (int k = 0; k < EPT; k++) acc0[k] = AR::acc_zero(), acc1[k] = AR::acc_zero();
    u32 terms = 0;
    for (u32 rr = 0; rr < a.n_rot; rr++) {
        const u64* key = a.key[rr] + (size_t)pi * N + base;
        const u32 gal = a.galois[rr];
        const u64* ptp = a.pt + ((size_t)rr * D + i) * N + base;
        u64 ptv[EPT];
        u32 idx[EPT];
#pragma unroll
        for (int k = 0; k < EPT; k++) {
            ptv[k] = a.pt ? __builtin_nontemporal_load(&ptp[k * 256]) : 1;
            idx[k] = eval_perm(base + k * 256, gal, tb.logN);
        }
        for (u32 j = 0; j < tb.dnum; j++) {
            const u64* k0 = key + ((size_t)j * 2 + 0) * Dkey * N;
            const u64* k1 = key + ((size_t)j * 2 + 1) * Dkey * N;
            const u64* src = j == own_digit ? a.ct + ((size_t)L + i) * N : a.dt + ((size_t)j * D + i) * N;
            u64 kv0[EPT], kv1[EPT], sv[EPT];
#pragma unroll
            for (int k = 0; k < EPT; k++) {
                kv0[k] = __builtin_nontemporal_load(&k0[k * 256]);
                kv1[k] = __builtin_nontemporal_load(&k1[k * 256]);
                sv[k] = src[idx[k]];
            }
#pragma unroll
            for (int k = 0; k < EPT; k++) {
                const T w = AR::premul(sv[k], ptv[k], m);
                AR::acc_mac(acc0[k], w, kv0[k], m);
                AR::acc_mac(acc1[k], w, kv1[k], m);
            }
            if ((++terms & 7) == 0) {
#pragma unroll
                for (int k = 0; k < EPT; k++) acc0[k] = AR::acc_fold(acc0[k], m), acc1[k] = AR::acc_fold(acc1[k], m);
            }
        }
        if (is_q) {
#pragma unroll
            for (int k = 0; k < EPT; k++) AR::acc_mac(acc0[k], AR::premul(bp[idx[k]], ptv[k], m), pmod, m);
            if ((++terms & 7) == 0) {
#pragma unroll
                for (int k = 0; k < EPT; k++) acc0[k] = AR::acc_fold(acc0[k], m), acc1[k] = AR::acc_fold(acc1[k], m);
            }
        }
    }
    const u32 sp = a.split;
    u64* o0 = (i < sp ? a.cq + (size_t)i * N : a.cp + (size_t)(i - sp) * N) + base;
    u64* o1 = (i < sp ? a.cq + ((size_t)sp + i) * N : a.cp + ((size_t)(D - sp) + (i - sp)) * N) + base;
#pragma unroll
    for (int k = 0; k < EPT; k++) {
        u64 r0 = AR::acc_canon(AR::acc_finish2(acc0[k], m), m), r1 = AR::acc_canon(AR::acc_finish2(acc1[k], m), m);
        if (a.accumulate) r0 = addmod(r0, o0[k * 256], pc.q), r1 = addmod(r1, o1[k * 256], pc.q);
        o0[k * 256] = r0;
        o1[k * 256] = r1;
    }
}

// ==================================================== baby-step giant-step accumulation and sums
// C[g][t][i] = sum_b pt[g][b][i] * R[b][t][i] on every limb i of the extended basis: the giant-step
// combinations of the baby-step rotations R_b (kept in the extended basis, times P).  Element-parallel;
// one workgroup per 256 * EPT slots of (limb, giant step).
struct BsgsMacArgs {
    const u64* rq;  // [n1][2][L][N]  q-limbs of R_b
    const u64* rp;  // [n1][2][K][N]  special limbs of R_b
    const u64* pt;  // [n2][n1][D][N]
    u64* cq;        // [n2][2][L][N]
    u64* cp;        // [n2][2][K][N]
    u32 n1, n2;
};

template <class AR, int EPT>
__global__ __launch_bounds__(256) void bsgs_mac_kernel(BsgsMacArgs a, Tables tb, LimbRun run) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, L = tb.L, K = tb.K, D = tb.D;
    const u32 chunks = N / (256 * EPT);
    // the giant steps of one (limb, slot range) share the R_b they read: adjacent on one XCD
    u32 rest, g;
    if (!xcd_decode(blockIdx.x, a.n2, run.count * chunks, rest, g)) return;
    const u32 i = run.first + rest / chunks, base = (rest % chunks) * (256 * EPT) + tid;
    const PrimeConst pc = tb.pc[tb.phys(i)];
    const typename AR::Mod m = AR::mod(pc);
    const bool is_q = i < L;
    T acc0[EPT], acc1[EPT];
    u128w w0[EPT], w1[EPT];
#pragma unroll
    for (int k = 0; k < EPT; k++) acc0[k] = AR::acc_zero(), acc1[k] = AR::acc_zero(), w0[k] = u128w{0, 0}, w1[k] = u128w{0, 0};
    for (u32 b = 0; b < a.n1; b++) {
        const u64* r0 = (is_q ? a.rq + (((size_t)b * 2 + 0) * L + i) * N : a.rp + (((size_t)b * 2 + 0) * K + (i - L)) * N) + base;
        const u64* r1 = (is_q ? a.rq + (((size_t)b * 2 + 1) * L + i) * N : a.rp + (((size_t)b * 2 + 1) * K + (i - L)) * N) + base;
        const u64* pp = a.pt + (((size_t)g * a.n1 + b) * D + i) * N + base;
#pragma unroll
        for (int k = 0; k < EPT; k++) {
            const u64 pv = __builtin_nontemporal_load(&pp[k * 256]);
            if constexpr (AR::is_fp) {
                acc0[k] += AR::premul(r0[k * 256], pv, m);
                acc1[k] += AR::premul(r1[k * 256], pv, m);
            } else {  // at most 64 products below 2^122 fit the 128-bit accumulator
                mac128(w0[k], r0[k * 256], pv);
                mac128(w1[k], r1[k * 256], pv);
            }
        }
        if constexpr (AR::is_fp) {
            if ((b & 7) == 7) {
#pragma unroll
                for (int k = 0; k < EPT; k++) acc0[k] = AR::acc_fold(acc0[k], m), acc1[k] = AR::acc_fold(acc1[k], m);
            }
        }
    }
    u64* o0 = (is_q ? a.cq + (((size_t)g * 2 + 0) * L + i) * N : a.cp + (((size_t)g * 2 + 0) * K + (i - L)) * N) + base;
    u64* o1 = (is_q ? a.cq + (((size_t)g * 2 + 1) * L + i) * N : a.cp + (((size_t)g * 2 + 1) * K + (i - L)) * N) + base;
#pragma unroll
    for (int k = 0; k < EPT; k++) {
        if constexpr (AR::is_fp) {
            o0[k * 256] = AR::acc_canon(AR::acc_finish(acc0[k], m), m);
            o1[k * 256] = AR::acc_canon(AR::acc_finish(acc1[k], m), m);
        } else {
            o0[k * 256] = reduce128(w0[k], pc.q, pc.qneg, pc.r2);
            o1[k * 256] = reduce128(w1[k], pc.q, pc.qneg, pc.r2);
        }
    }
}

// out[l][n] = sum_g in[g][l][n] mod q_l over n_limbs limbs per item (limb l uses prime l % L).
__global__ __launch_bounds__(256) void sum_instances_kernel(const u64* __restrict__ in, u64* __restrict__ out,
                                                            const PrimeConst* pcs, u32 logN, u32 L, u32 n_limbs, u32 n_g) {
    const u32 N = 1u << logN;
    const u32 n = blockIdx.x * 256 + threadIdx.x, l = blockIdx.y;
    const u64 q = pcs[l % L].q;
    u64 acc = 0;
    for (u32 g = 0; g < n_g; g++) acc = addmod(acc, in[((size_t)g * n_limbs + l) * N + n], q);
    out[(size_t)l * N + n] = acc;
}

// ======================================================================== final combine
// ks_t[i] = (c'_t[i] - NTT(conv_t)[i]) * P^-1 mod q_i, the NTT's second pass done here, then
//   FIN_KS     : out[inst][t][i] = ks
//   FIN_HOISTED: out[t][i] (+)= sum_r pt_r[i] * (ks_r + (t == 0 ? sigma_{g_r}(b) : 0)); work item (i, tile, t)
// (HMult, HRot and the plain key switch end inside the inner-product kernel, which also adds the tensor
// terms or sigma_g(b).)  The numbering keeps kernel names stable.
enum FinalMode { FIN_KS = 0, FIN_HOISTED = 3 };
struct FinalArgs {
    const u64* cq;   // [g][2][L][N] canonical
    const u64* cv;   // [g][2][L][N] raw forward-lazy (first pass done)
    const u64* ct1;  // HOISTED: ct
    const u64* pt;   // HOISTED: plaintexts of this chunk [n_rot][L][N]
    u64* out;
    u32 galois[CKKS_ROT_CHUNK];
    u32 n_inst;      // batch (or 2 for HOISTED: the component t)
    u32 n_rot;       // HOISTED
    u32 accumulate;  // HOISTED: add to what out already holds
    u32 cq_L;        // limbs per component of cq (L, or L + 1 when cq is a ciphertext about to lose its last limb)
};

template <class AR, int A, int MODE>
__device__ __forceinline__ void ks_final_body(const FinalArgs& a, const Tables& tb, u64* lds, u32 i, u32 tile, u32 inst) {
    typedef typename AR::T T;
    const u32 N = 1u << tb.logN, tid = threadIdx.x, e0 = tid % 16, ch = tid / 16, r = tile * 16 + ch;
    const u32 L = tb.L;
    const PrimeConst pc = tb.pc[i];
    const typename AR::Mod m = AR::mod(pc);
    const PinvConst pinv = tb.pinv[i];
    const u64* ti = tb.tw_int + (size_t)i * 4 * N;
    const double* tf = tb.tw_fp + (size_t)i * 2 * N;
    u64* lrow = lds + ch * 272;
    const u32 row_off = r * 256;
    const u64 q = pc.q;
    // The converted part leaves its second forward pass in layout CP: c', plaintexts and results move with 16-byte
    // accesses, and sigma_g(b) comes as a whole source row permuted in LDS (gather_row_cp).
    // FP64 pipe (magnitudes in units of q): v <= 5.2, c' - v <= 6.2, ks = (c' - v) * P^-1 <= 2.9,
    // every added product of canonical operands <= 0.875; everything is canonicalised before the store.
    if (MODE == FIN_HOISTED) {
        const u32 t = inst;
        double facc[AR::is_fp ? 16 : 1];
        u128w iacc[AR::is_fp ? 1 : 16];
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if constexpr (AR::is_fp) facc[k] = 0.0;
            else iacc[k] = u128w{0, 0};
        }
        for (u32 rr = 0; rr < a.n_rot; rr++) {
            T v[16];
            const u64* p = a.cv + (((size_t)rr * 2 + t) * L + i) * N + row_off;
#pragma unroll
            for (int k = 0; k < 16; k++) v[k] = AR::from_raw(__builtin_nontemporal_load(&p[k * 16 + e0]));
            NttCore<AR, A>::fwd_contig(v, lrow, e0, r, ti, tf, N, m);
            exchange_cb_to_cp<AR>(v, lrow, e0);
            // one operand stream at a time: c', then sigma_g(b), then the plaintext (16 words each)
            T ks[16];
            {
                u64 c[16];
                load_row_cp<true>(a.cq + (((size_t)rr * 2 + t) * L + i) * N + row_off, e0, c);
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    if constexpr (AR::is_fp) ks[k] = FpAr::mulmod_lazy(u64_to_f64(c[k]) - v[k], pinv.d, FpAr::mod(pc));
                    else ks[k] = mul_shoup(submod(c[k], AR::canon_fwd(v[k], m), q), pinv.w, pinv.wp, q);
                }
            }
            if (t == 0) {
                u64 bw[16];
                gather_row_cp(a.ct1 + (size_t)i * N, row_off, a.galois[rr], tb.logN, lrow, e0, bw);
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    if constexpr (AR::is_fp) ks[k] += u64_to_f64(bw[k]);
                    else ks[k] = addmod(ks[k], bw[k], q);
                }
            }
            {
                u64 ptw[16];
                load_row_cp<true>(a.pt + ((size_t)rr * L + i) * N + row_off, e0, ptw);
#pragma unroll
                for (int k = 0; k < 16; k++) {
                    // FP64: reduced to <= q/2 so that the at most 8 products accumulated between folds stay below 6 q
                    if constexpr (AR::is_fp) facc[k] += FpAr::mulmod_lazy(FpAr::reduce(ks[k], FpAr::mod(pc)), u64_to_f64(ptw[k]), FpAr::mod(pc));
                    else mac128(iacc[k], ks[k], ptw[k]);
                }
            }
            if constexpr (AR::is_fp) {
                if ((rr & 7) == 7) {
#pragma unroll
                    for (int k = 0; k < 16; k++) facc[k] = FpAr::reduce(facc[k], FpAr::mod(pc));
                }
            }
        }
        u64* o = a.out + ((size_t)t * L + i) * N + row_off;
        u64 prev[16], res[16];
        if (a.accumulate) load_row_cp<false>(o, e0, prev);
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if constexpr (AR::is_fp) {
                double x = facc[k];
                if (a.accumulate) x += u64_to_f64(prev[k]);
                res[k] = FpAr::canon(x, FpAr::mod(pc));
            } else {
                res[k] = reduce128(iacc[k], q, pc.qneg, pc.r2);
                if (a.accumulate) res[k] = addmod(res[k], prev[k], q);
            }
        }
        store_row_cp(o, e0, res);
        return;
    }
#pragma unroll
    for (int t = 0; t < 2; t++) {
        T v[16];
        const u64* p = a.cv + (((size_t)inst * 2 + t) * L + i) * N + row_off;
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = AR::from_raw(__builtin_nontemporal_load(&p[k * 16 + e0]));
        NttCore<AR, A>::fwd_contig(v, lrow, e0, r, ti, tf, N, m);
        exchange_cb_to_cp<AR>(v, lrow, e0);
        u64 c[16], res[16];
        load_row_cp<true>(a.cq + (((size_t)inst * 2 + t) * a.cq_L + i) * N + row_off, e0, c);
#pragma unroll
        for (int k = 0; k < 16; k++) {
            if constexpr (AR::is_fp) {
                const FpAr::Mod fm = FpAr::mod(pc);
                res[k] = FpAr::canon(FpAr::mulmod_lazy(u64_to_f64(c[k]) - v[k], pinv.d, fm), fm);
            } else {
                res[k] = mul_shoup(submod(c[k], AR::canon_fwd(v[k], m), q), pinv.w, pinv.wp, q);
            }
        }
        store_row_cp(a.out + (((size_t)inst * 2 + t) * L + i) * N + row_off, e0, res);
    }
}

template <class AR, int A, int MODE>
__global__ __launch_bounds__(256, MODE == FIN_HOISTED ? (AR::is_fp ? 3 : 2) : 4) void ks_final_kernel(FinalArgs a, Tables tb, LimbRun run) {
    __shared__ u64 lds[NTT_LDS_WORDS];
    constexpr u32 TILES = (1u << A) / 16;
    u32 group, inst;
    if (!xcd_decode(blockIdx.x, a.n_inst, run.count * TILES, group, inst)) return;
    ks_final_body<AR, A, MODE>(a, tb, lds, run.first + group / TILES, group % TILES, inst);
}

// ================================================== stand-alone coefficient-form base conversions
// in [b][L][N] coeff -> out [b][dnum][D][N].  grid (N/256, dnum, batch).
template <int ALPHA>
__global__ __launch_bounds__(256) void modup_kernel(const u64* __restrict__ in, u64* __restrict__ out, Tables tb) {
    const u32 N = 1u << tb.logN, L = tb.L, D = tb.D;
    const u32 n = blockIdx.x * 256 + threadIdx.x, j = blockIdx.y, b = blockIdx.z;
    const u64* src = in + ((size_t)b * L + (size_t)j * ALPHA) * N + n;
    u64* dst = out + ((size_t)b * tb.dnum + j) * D * N + n;
    const u32 ns = (j + 1) * ALPHA <= L ? ALPHA : L - j * ALPHA;  // the last digit may be shorter
    u64 y[ALPHA];
#pragma unroll
    for (int ii = 0; ii < ALPHA; ii++) {
        y[ii] = 0;
        if ((u32)ii < ns) {
            const u32 i = j * ALPHA + ii;
            const u64 x = src[(size_t)ii * N];
            dst[(size_t)i * N] = x;
            y[ii] = mul_shoup(x, tb.up_hatinv[2 * i], tb.up_hatinv[2 * i + 1], tb.pc[i].q);
        }
    }
    const u64* chat = tb.up_chat + (size_t)j * ALPHA * D;
    for (u32 t = 0; t < D; t++) {
        if (t >= j * ALPHA && t < j * ALPHA + ns) continue;
        u128w acc = {0, 0};
        const PrimeConst pc = tb.pc[t];
#pragma unroll
        for (int ii = 0; ii < ALPHA; ii++) {
            if ((u32)ii < ns) mac128(acc, y[ii], chat[(size_t)ii * D + t]);
            if (ALPHA > 8 && ((ii & 7) == 7 || ii + 1 == ALPHA)) acc.hi = csub(acc.hi, pc.q);  // keeps acc < q * 2^64
        }
        dst[(size_t)t * N] = redc(acc, pc.q, pc.qneg);
    }
}

// in [g][D][N] coeff -> out [g][L][N] = (in_i - conv_i) * P^-1.  grid (N/256, groups).
template <int KK>
__global__ __launch_bounds__(256) void moddown_kernel(const u64* __restrict__ in, u64* __restrict__ out, Tables tb) {
    const u32 N = 1u << tb.logN, L = tb.L, D = tb.D;
    const u32 n = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
    const u64* src = in + (size_t)g * D * N + n;
    u64* dst = out + (size_t)g * L * N + n;
    u64 y[KK];
#pragma unroll
    for (int k = 0; k < KK; k++)
        y[k] = mul_shoup(src[(size_t)(L + k) * N], tb.dn_hatinv[2 * k], tb.dn_hatinv[2 * k + 1], tb.pc[L + k].q);
    for (u32 i = 0; i < L; i++) {
        u128w acc = {0, 0};
        const PrimeConst pc = tb.pc[i];
#pragma unroll
        for (int k = 0; k < KK; k++) {
            mac128(acc, y[k], tb.dn_chat[(size_t)k * L + i]);
            if (KK > 8 && ((k & 7) == 7 || k + 1 == KK)) acc.hi = csub(acc.hi, pc.q);  // keeps acc < q * 2^64
        }
        const u64 conv = redc(acc, pc.q, pc.qneg);
        const PinvConst pi = tb.pinv[i];
        dst[(size_t)i * N] = mul_shoup(submod(src[(size_t)i * N], conv, pc.q), pi.w, pi.wp, pc.q);
    }
}

// ------------------------------------------------------------------------ automorphism
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

// -------------------------------------------------------------------- limb-wise arithmetic
// out[g][l][n] = a[g][l][n] (op) b[g % b_period][l][n] mod prime (prime_first + l); two words per lane
// (16-byte accesses).  out may be a or b themselves: every lane reads its words before it writes them.
enum PointwiseOp { PW_ADD = 0, PW_SUB = 1, PW_MUL = 2, PW_MAC = 3 };
template <int OP>
__global__ __launch_bounds__(256) void pointwise_kernel(const u64* a, const u64* b, u64* out, const PrimeConst* pcs,
                                                        u32 logN, u32 n_limbs, u32 prime_first, u32 b_period) {
    const u32 N = 1u << logN;
    const u32 n = (blockIdx.x * 256 + threadIdx.x) * 2;
    const size_t la = ((size_t)blockIdx.z * n_limbs + blockIdx.y) * N + n;
    const size_t lb = ((size_t)(blockIdx.z % b_period) * n_limbs + blockIdx.y) * N + n;
    const PrimeConst pc = pcs[prime_first + blockIdx.y];
    const ulonglong2 av = *reinterpret_cast<const ulonglong2*>(a + la);
    const ulonglong2 bv = *reinterpret_cast<const ulonglong2*>(b + lb);
    ulonglong2 r;
    if (OP == PW_ADD) {
        r.x = addmod(av.x, bv.x, pc.q), r.y = addmod(av.y, bv.y, pc.q);
    } else if (OP == PW_SUB) {
        r.x = submod(av.x, bv.x, pc.q), r.y = submod(av.y, bv.y, pc.q);
    } else {
        r.x = mulmod_var(av.x, bv.x, pc.q, pc.qneg, pc.r2), r.y = mulmod_var(av.y, bv.y, pc.q, pc.qneg, pc.r2);
        if (OP == PW_MAC) {
            const ulonglong2 ov = *reinterpret_cast<const ulonglong2*>(out + la);
            r.x = addmod(r.x, ov.x, pc.q), r.y = addmod(r.y, ov.y, pc.q);
        }
    }
    *reinterpret_cast<ulonglong2*>(out + la) = r;
}
