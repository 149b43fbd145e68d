/*
 * ckks_mi355x.h -- C ABI of the MI355X (gfx950) RNS-CKKS key-switch library.
 *
 * Scope: the polynomial kernels of the GPU RNS-CKKS library described in the
 * paper's Section 2 ("A GPU Library Supporting RNS-CKKS") -- NTT and base
 * conversion, the kernels it names as the major ones -- and the thin slice of
 * HE operations built from them (HMult with relinearisation, rotation; Table 1
 * and Section 4).  The paper defers the definition of each step to the full-RNS
 * CKKS scheme it cites; the definitions used here are restated with every
 * entry point.
 *
 * Object (Section 2): a polynomial of Z_Q[X]/(X^N+1) is an L x N matrix of
 * 64-bit words, one row ("limb") per RNS prime, stored limb-major.
 *
 * Conventions that hold for EVERY call
 *   - every data pointer named d_* is DEVICE memory owned by the caller,
 *     contiguous, 16-byte aligned, uint64 words, layout [...][limb][N];
 *     pointers named h_* are HOST memory read during the call only.
 *   - residues are canonical, in [0, prime), on entry and on exit.
 *   - prime order: q_0 .. q_{L-1} (ciphertext limbs), then p_0 .. p_{K-1}
 *     (special limbs).  D = L + K.  alpha = L / dnum; digit j owns the limbs
 *     j*alpha .. (j+1)*alpha-1.
 *   - a ciphertext is [2][L][N] in evaluation form: index 0 = c0 (b),
 *     1 = c1 (a); it decrypts as c0 + c1*s.
 *   - a switching key is [dnum][2][D][N] in evaluation form.
 *   - evaluation form of limb i: slot j holds the polynomial evaluated at
 *     psi_i^(2*bitrev(j)+1) (bit-reversed order), psi_i a primitive 2N-th root
 *     of unity modulo prime i; coefficient form is natural order.
 *   - all work is enqueued on `stream` (a hipStream_t passed as void*; NULL =
 *     the default stream) and is asynchronous; the caller synchronises.
 *   - input and output buffers must not overlap unless "in place" is stated.  The calls that take a
 *     workspace check this on the host and return CKKS_EINVAL, launching nothing, when an output shares
 *     bytes with a ciphertext / plaintext input or when the workspace shares bytes with either (the
 *     kernels re-read inputs after the first output words are written, so such a call would return
 *     wrong words without any error); keys are read-only and are not part of that check.
 *   - the library allocates no device memory: tables and workspace are caller
 *     buffers sized by ckks_table_bytes / ckks_workspace_bytes, 256-byte aligned.
 *   - return value: CKKS_OK or a negative error code; nothing throws or aborts.
 *     ckks_last_error() gives a message for the last failing call on a context.
 *   - digits hold alpha = ceil(L / dnum) consecutive limbs; the last digit is shorter when dnum does not
 *     divide L (dnum must be the digit count that this size gives: ceil(L / alpha) = dnum).  The calls
 *     without a level work on full-level operands (all L limbs present); the calls ending in _at, ckks_rescale and the merged-rescale calls take the number
 *     of active limbs as `level` and use the same context, tables and full-level keys.
 *   - the calls may be captured in a HIP graph: they only launch kernels (no allocation, no
 *     memset), provided profiling is off.
 */
#ifndef CKKS_MI355X_H
#define CKKS_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKKS_OK 0
#define CKKS_EINVAL (-1)       /* null / misaligned pointer, size out of range, bad Galois element */
#define CKKS_EUNSUPPORTED (-2) /* shape outside what the kernels are built for */
#define CKKS_EHIP (-3)         /* a HIP runtime call failed */
#define CKKS_ENOMEM (-4)       /* caller's table / workspace buffer too small */

/* selectors for ckks_workspace_bytes */
#define CKKS_OP_NTT 0
#define CKKS_OP_MODUP 1
#define CKKS_OP_MODDOWN 2
#define CKKS_OP_AUTOMORPH 3
#define CKKS_OP_KEYSWITCH 4
#define CKKS_OP_HMULT_RELIN 5
#define CKKS_OP_HROT 6
#define CKKS_OP_HROT_HOISTED_MAC 7
#define CKKS_OP_RESCALE 8
#define CKKS_OP_HROT_DH_MAC 9

/* operations of ckks_pointwise */
#define CKKS_PW_ADD 0 /* out = a + b */
#define CKKS_PW_SUB 1 /* out = a - b */
#define CKKS_PW_MUL 2 /* out = a * b */
#define CKKS_PW_MAC 3 /* out = out + a * b */

/* limits of this build */
#define CKKS_MIN_LOGN 12
#define CKKS_MAX_LOGN 16
#define CKKS_MAX_PRIMES 128 /* L + K */
#define CKKS_MAX_DIGIT 16  /* alpha and K */
#define CKKS_MAX_PRIME_BITS 61
#define CKKS_STATIC_SCRATCH_BYTES (32u << 20) /* per-GPU scratch of ckks_rescale_static */
#define CKKS_ROTATIONS_PER_LAUNCH 16 /* instances with their own key that one launch takes (chunking of rotation batches) */

typedef struct ckks_ctx ckks_ctx;

/* Bytes of device memory ckks_ctx_create needs for twiddle and constant tables. */
int ckks_table_bytes(uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, size_t* bytes);

/*
 * Build a context: validates the parameter set, derives on the host every
 * per-prime table (powers of psi in bit-reversed order for the forward and the
 * inverse transform, base-conversion constants for every digit and for the
 * special basis) and copies them into d_tables.
 *   h_primes : L+K primes, each = 1 mod 2N and < 2^61, pairwise distinct.
 *   h_psi    : L+K primitive 2N-th roots, or NULL = the numerically smallest
 *              psi with psi^N = -1 for every prime.
 *   K may be 0 (transform-only context; key-switch calls then return
 *   CKKS_EUNSUPPORTED).  Returns after the copy has completed.
 *   Shape limits: CKKS_MIN_LOGN <= logN <= CKKS_MAX_LOGN, L + K <= CKKS_MAX_PRIMES,
 *   alpha = ceil(L / dnum) <= CKKS_MAX_DIGIT with ceil(L / alpha) = dnum, and K <= CKKS_MAX_DIGIT
 *   (else CKKS_EUNSUPPORTED).
 * Ownership: the context keeps d_tables in use until ckks_ctx_destroy; the
 * caller frees it afterwards.
 */
int ckks_ctx_create(ckks_ctx** out, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                    const uint64_t* h_primes, const uint64_t* h_psi, void* d_tables, size_t table_bytes,
                    void* stream);

/* Frees host state only. NULL is allowed.  A context (its error string, profiling state, optional second
 * stream) is not synchronised: use it from one host thread at a time; device work of different calls on
 * different streams may overlap only if they use different workspaces. */
void ckks_ctx_destroy(ckks_ctx* ctx);

/* Message of the last error on this context (owned by the context; "" if none). */
const char* ckks_last_error(const ckks_ctx* ctx);

/* The root of unity in use for prime index i (0 on a bad index). */
uint64_t ckks_ctx_psi(const ckks_ctx* ctx, uint32_t i);

/* Bytes of workspace the given op needs for `batch_or_nrot` (batch size; number of rotations
 * for CKKS_OP_HROT_HOISTED_MAC and CKKS_OP_HROT_DH_MAC).  0 for ops that need none.  The merged-rescale
 * calls use the size of their un-merged counterpart; ckks_hrot_multi_at that of CKKS_OP_HROT for
 * min(batch, CKKS_ROTATIONS_PER_LAUNCH); ckks_lintrans_bsgs_at has its own query. */
int ckks_workspace_bytes(const ckks_ctx* ctx, int op, uint32_t batch_or_nrot, size_t* bytes);

/* The same for an operation at `level` active q-limbs (1 <= level <= L; for CKKS_OP_RESCALE the level of
 * the input).  Never more than the full-level figure, so one full-level workspace serves every level. */
int ckks_workspace_bytes_at(const ckks_ctx* ctx, int op, uint32_t level, uint32_t batch_or_nrot, size_t* bytes);

/*
 * Forward negacyclic NTT, in place, batched (Section 2: "NTT", a major kernel).
 *   d_x : [batch][n_limbs][N]; limb l is reduced modulo prime (prime_first + l).
 *   X^[j] = sum_t x_t * psi^(t*(2*bitrev(j)+1)) mod prime: natural-order coefficients in,
 *   bit-reversed evaluation order out.
 */
int ckks_ntt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch, void* stream);

/* Inverse of ckks_ntt (includes the factor N^-1): evaluation form in, natural-order coefficients out. */
int ckks_intt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch, void* stream);

/*
 * ModUp: digit decomposition + fast base conversion (Section 2: "base conversion"), coefficient form.
 *   d_in  : [batch][L][N]     d_out : [batch][dnum][D][N]
 *   For digit j and coefficient n, with C_j the digit's primes and Q_j their product:
 *     y_i = x_i * [(Q_j/q_i)^-1]_{q_i} mod q_i   (canonical),
 *     out[j][t] = sum_{i in C_j} y_i * ((Q_j/q_i) mod m_t)  mod m_t    for every prime m_t outside C_j,
 *     out[j][t] = x_t                                                   for t in C_j.
 *   No correction of the overflow multiple of Q_j is applied.
 */
int ckks_modup(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream);

/*
 * ModDown: division by P = p_0*...*p_{K-1} with floor-type rounding, coefficient form.
 *   d_in : [batch][D][N]      d_out : [batch][L][N]
 *   out_i = (in_i - Conv_{P -> q_i}(in restricted to the special limbs)) * [P^-1]_{q_i}  mod q_i,
 *   Conv being the same uncorrected fast base conversion as in ModUp with source basis p_0..p_{K-1}.
 */
int ckks_moddown(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream);

/*
 * Galois automorphism sigma_g : X -> X^g (the map behind homomorphic rotation, Section 4).
 *   d_in, d_out : [batch][n_limbs][N], limb l modulo prime (prime_first + l); galois odd, < 2N.
 *   eval_domain = 0: coefficient form, out[(t*g mod 2N) mod N] = +-in[t] (minus when t*g mod 2N >= N).
 *   eval_domain = 1: evaluation form, out[j] = in[j'] with 2*bitrev(j')+1 = g*(2*bitrev(j)+1) mod 2N.
 */
int ckks_automorph(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t prime_first, uint32_t n_limbs,
                   uint32_t galois, int eval_domain, uint32_t batch, void* stream);

/*
 * Limb-wise arithmetic on residue matrices: the L x N element-parallel operations of Section 3 (addition of
 * polynomials), and in evaluation form the products behind the multiplication of a ciphertext by a plaintext
 * that the convolutions of Section 5 accumulate.
 *   d_a, d_out : [batch][n_limbs][N]      d_b : [b_period][n_limbs][N], 1 <= b_period <= batch
 *   out[g][l][n] = a[g][l][n] (op) b[g % b_period][l][n]  mod prime (prime_first + l),
 *   op = CKKS_PW_ADD | CKKS_PW_SUB | CKKS_PW_MUL, or CKKS_PW_MAC: out = out + a * b.
 *   b_period = batch pairs the operands one to one; b_period = 1 applies one plaintext to every polynomial
 *   of a (both components of every ciphertext of a batch).  Residues canonical on entry and exit.  d_out may be
 *   d_a or d_b themselves (same address), but may not overlap them otherwise.  No workspace.
 */
int ckks_pointwise(ckks_ctx* ctx, int op, const uint64_t* d_a, const uint64_t* d_b, uint64_t* d_out,
                   uint32_t prime_first, uint32_t n_limbs, uint32_t batch, uint32_t b_period, void* stream);

/*
 * Hybrid key switch (the step inside HMult and rotation; Table 1 measures HMult):
 *   x = INTT(d);  dt = ModUp(x);  Dh_j = NTT(dt_j) on all D limbs;
 *   c'_t[i] = sum_j Dh_j[i] * key[j][t][i] mod m_i  (t = 0,1);
 *   out_t = NTT(ModDown(INTT(c'_t))).
 *   d_d : [batch][L][N] eval;  d_key : [dnum][2][D][N] eval (shared by the batch);  d_out : [batch][2][L][N] eval.
 */
int ckks_keyswitch(ckks_ctx* ctx, const uint64_t* d_d, const uint64_t* d_key, uint64_t* d_out, uint32_t batch,
                   void* d_ws, size_t ws_bytes, void* stream);

/*
 * HMult with relinearisation, no rescale (Table 1 "HMult"):
 *   d0 = b1*b2, d1 = a1*b2 + a2*b1, d2 = a1*a2 (limb-wise, evaluation form);
 *   out = (d0 + ks_0, d1 + ks_1), ks = KeySwitch(d2, evk).
 *   d_ct1, d_ct2, d_out : [batch][2][L][N];  d_evk : [dnum][2][D][N].
 */
int ckks_hmult_relin(ckks_ctx* ctx, const uint64_t* d_ct1, const uint64_t* d_ct2, const uint64_t* d_evk,
                     uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Homomorphic rotation by the Galois element g (Section 4: rotations dominate convolution time):
 *   out = (sigma_g(b) + ks_0, ks_1), ks = KeySwitch(sigma_g(a), rk_g), sigma_g on evaluation form.
 *   d_ct, d_out : [batch][2][L][N];  d_rk : [dnum][2][D][N].
 */
int ckks_hrot(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t galois, const uint64_t* d_rk, uint64_t* d_out,
              uint32_t batch, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Hoisted rotate-multiply-accumulate (the convolution / linear-transform shape of Section 4):
 *   Dh_j = NTT(ModUp(INTT(a))_j) once; then for every rotation r
 *     c'_t = sum_j sigma_{g_r}(Dh_j) * rk_r[j][t];  ks = NTT(ModDown(INTT(c')));
 *     R_r = (sigma_{g_r}(b) + ks_0, ks_1);   out += pt_r * R_r  (both components).
 *   d_ct : [2][L][N];  h_galois : n_rot Galois elements (host);  h_rk_ptrs : host array of n_rot device
 *   pointers, each a [dnum][2][D][N] key;  d_pt : [n_rot][L][N] eval;  d_out : [2][L][N] (overwritten).
 */
int ckks_hrot_hoisted_mac(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                          const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out, void* d_ws,
                          size_t ws_bytes, void* stream);

/*
 * Levels below L (Section 4: every layer of the CNN consumes multiplicative levels, so most
 * operations run on ciphertexts that have already lost limbs).  A ciphertext at `level` = ell
 * (1 <= ell <= L) holds the limbs q_0..q_{ell-1}: [batch][2][ell][N].  The `_at` calls are the
 * operations above on that basis with the SAME full-level keys [dnum][2][L+K][N]:
 *   extended basis q_0..q_{ell-1}, p_0..p_{K-1};  ceil(ell/alpha) digits, digit j = limbs
 *   j*alpha .. min((j+1)*alpha, ell)-1, the last digit possibly partial (its conversion constants are
 *   those of the limbs it really has);  the key is read on the active and the special limbs of these
 *   digits only;  ModDown divides by P as before.
 * level = L gives exactly ckks_keyswitch / ckks_hmult_relin / ckks_hrot / ckks_hrot_hoisted_mac.
 * Shapes: as the full-level calls with L replaced by ell everywhere except in the keys
 * (d_pt : [n_rot][ell][N]).  level outside 1..L: CKKS_EINVAL.
 */
int ckks_keyswitch_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_d, const uint64_t* d_key, uint64_t* d_out,
                      uint32_t batch, void* d_ws, size_t ws_bytes, void* stream);
int ckks_hmult_relin_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct1, const uint64_t* d_ct2,
                        const uint64_t* d_evk, uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes,
                        void* stream);
int ckks_hrot_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t galois, const uint64_t* d_rk,
                 uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream);
int ckks_hrot_hoisted_mac_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot,
                             const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt,
                             uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Rescale (the step that consumes a level, Section 4): divide by the last active prime q = q_{level-1}
 * and drop its limb, floor type like ModDown.  With X in [0, Q_level) the value of a coefficient the
 * result is (X - [X]_q) / q modulo Q_{level-1}, [.]_q the canonical representative in [0, q):
 *   out_i = (in_i - NTT_i([INTT(in_{level-1})]_q mod q_i)) * [q^-1]_{q_i}  mod q_i,   i < level-1.
 *   d_ct : [batch][2][level][N] eval;  d_out : [batch][2][level-1][N] eval (must not overlap d_ct);
 *   2 <= level <= L.  Works on contexts without special primes as well.
 */
int ckks_rescale(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint64_t* d_out, uint32_t batch, void* d_ws,
                 size_t ws_bytes, void* stream);

/*
 * ckks_rescale for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands, same result words as
 * ckks_rescale; the workspace is a static device array inside the library, CKKS_STATIC_SCRATCH_BYTES
 * (32 MiB) on every GPU the library is loaded on, held until the process ends.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine) and only launches kernels.
 *   Limit: batch * 2 * level * N * 8 bytes <= CKKS_STATIC_SCRATCH_BYTES (N = 2^16: batch * level <= 32, e.g. one
 *   ciphertext at level 32, two at level 16); larger requests return CKKS_ENOMEM and launch nothing.
 *   The device current at the call must be the one the context was created on (else CKKS_EINVAL).
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams,
 *   different contexts, different threads) race on it and must be ordered by the caller.  Nothing needs
 *   clearing between calls: every scratch word a call reads it has written first.
 */
int ckks_rescale_static(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint64_t* d_out, uint32_t batch,
                        void* stream);

/*
 * Double-hoisted rotate-multiply-accumulate (the linear-transform evaluation of the bootstrapping
 * the paper adopts, Section 2 / Table 1 "Boot"): besides sharing the decomposition, the plaintext
 * products are summed in the extended basis and ONE ModDown is applied to the sum:
 *   Dh_j as in ckks_hrot_hoisted_mac;  c'_{r,t} = sum_j sigma_{g_r}(Dh_j) * rk_r[j][t]  on all ell+K limbs;
 *   C_t = sum_r pt_r * c'_{r,t};   out_t = NTT(ModDown(INTT(C_t))) + (t == 0 ? sum_r pt_r * sigma_{g_r}(b) : 0).
 *   d_pt : [n_rot][ell+K][N] eval, the plaintext modulo every prime of the level's extended basis
 *   (q_0..q_{ell-1}, then p_0..p_{K-1});  everything else as ckks_hrot_hoisted_mac(_at).
 * Not bit-identical to the singly hoisted call (ModDown of a sum is not the sum of ModDowns); one
 * rotation with the all-ones plaintext gives exactly that rotation's singly hoisted result.
 */
int ckks_hrot_dh_mac(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                     const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out, void* d_ws,
                     size_t ws_bytes, void* stream);
int ckks_hrot_dh_mac_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                        const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out, void* d_ws,
                        size_t ws_bytes, void* stream);

/*
 * ModDown merged with the rescale that follows it (Section 4: every multiplication of the CNN is followed
 * by a rescale): one floor-type division by P * q_{level-1}.  The last active limb joins the special limbs
 * as a source of the conversion:  S = {q_{level-1}, p_0..p_{K-1}}, PS its product,
 *   out_i = (C_i - Conv_{S -> q_i}(C restricted to S)) * [PS^-1]_{q_i}  mod q_i,   i < level-1.
 * ckks_hmult_relin_rescale_at:  C_t = c'_t + P * d_t on the q-limbs (d_0 = b1*b2, d_1 = a1*b2 + a2*b1, c' the
 *   inner product of ckks_hmult_relin_at), C_t = c'_t on the special limbs;
 *   d_ct1, d_ct2 : [batch][2][level][N];  d_out : [batch][2][level-1][N].
 * ckks_hrot_dh_mac_rescale_at:  C_t of ckks_hrot_dh_mac_at with P * sum_r pt_r * sigma_{g_r}(b) added to C_0 on
 *   the q-limbs;  d_out : [2][level-1][N];  everything else as ckks_hrot_dh_mac_at.
 * As integers the results are floor(X / PS) - u, 0 <= u <= K: within K+1 of, but not bit-identical to, the
 * un-merged call followed by ckks_rescale.  2 <= level <= L.  Workspace: as the un-merged call at that level.
 */
int ckks_hmult_relin_rescale_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct1, const uint64_t* d_ct2,
                                const uint64_t* d_evk, uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes,
                                void* stream);
int ckks_hrot_dh_mac_rescale_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot,
                                const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt,
                                uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Rotations of a batch of ciphertexts, instance b by the Galois element h_galois[b] with the key h_rk_ptrs[b]
 * (host arrays of `batch` entries): out[b] = ckks_hrot_at(level, ct[b], h_galois[b], rk_b).  Issued in chunks of
 * CKKS_ROTATIONS_PER_LAUNCH instances; the workspace of CKKS_OP_HROT for min(batch, CKKS_ROTATIONS_PER_LAUNCH) at that
 * level suffices.
 */
int ckks_hrot_multi_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, const uint32_t* h_galois,
                       const uint64_t* const* h_rk_ptrs, uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes,
                       void* stream);

/*
 * Baby-step giant-step linear transform (the shape of the CoeffToSlot / SlotToCoeff stages of the
 * bootstrapping the paper adopts, Table 1 "Boot"; diagonals are given as ready plaintext polynomials):
 *   inner_g = double-hoisted rotate-multiply-accumulate of ct over the n1 baby rotations with the
 *             plaintexts pt[g][0..n1)                         (the definition of ckks_hrot_dh_mac_at),
 *   out     = sum_g HRot(inner_g, giant rotation g)           (the definition of ckks_hrot_at; limb-wise sum).
 * Every rotation, identities (Galois element 1) included, is a key switch with the key given for it.
 *   d_ct : [2][level][N];  d_pt : [n2][n1][level+K][N] on the level's extended basis;  d_out : [2][level][N];
 *   h_*_galois / h_*_rk_ptrs : host arrays (n1 baby, n2 giant) of Galois elements and device key pointers;
 *   1 <= n1, n2 <= 64.  The baby rotations are computed once, kept in the extended basis and shared by all
 *   giant steps; results are identical to composing the two calls above.
 */
int ckks_lintrans_bsgs_workspace_bytes(const ckks_ctx* ctx, uint32_t level, uint32_t n1, uint32_t n2, size_t* bytes);
int ckks_lintrans_bsgs_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n1, const uint32_t* h_baby_galois,
                          const uint64_t* const* h_baby_rk_ptrs, uint32_t n2, const uint32_t* h_giant_galois,
                          const uint64_t* const* h_giant_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out, void* d_ws,
                          size_t ws_bytes, void* stream);

/*
 * Optional two-stream execution inside one call.  Off by default: every kernel of a call runs on the
 * caller's stream in order.  With on != 0 a call may put part of its launches on a second stream owned by
 * the context, ordered by events (both streams at default priority): ckks_keyswitch, ckks_hmult_relin,
 * ckks_hrot and their _at / _multi / _rescale forms run the ModUp conversion of the floating-point-arithmetic
 * limbs there, beside the inner product and ModDown conversion of the integer-arithmetic limbs (primes of
 * 50 bits and more, normally the special limbs); the hoisted, double-hoisted and baby-step giant-step calls
 * run the launches on integer-arithmetic limbs there, beside those on floating-point-arithmetic limbs.
 * Needs both classes of primes in the chain, otherwise nothing changes.  Results are identical; the call
 * still completes in stream order on the caller's stream.  Not to be changed while a call of this context
 * is being issued.
 */
int ckks_set_overlap(ckks_ctx* ctx, int on);

/*
 * Measurement support (no part of the method): per-kernel timing with HIP events.
 * ckks_profile_enable(ctx, 1) clears the counters and makes every later kernel launch of this
 * context be bracketed by two HIP events recorded on the launch stream; (ctx, 0) stops that.
 * ckks_profile_read waits for the recorded events and returns, for the index-th kernel
 * instantiation seen since the counters were cleared: its name as a profiler prints it (owned by
 * the context, valid until the next ckks_profile_enable), the number of launches, their summed
 * duration in milliseconds and their summed algorithmic bytes (the words each launch must read
 * and write once, tables excluded).  Returns CKKS_EINVAL once index is past the last entry.
 * Any output pointer may be NULL.
 */
int ckks_profile_enable(ckks_ctx* ctx, int on);
int ckks_profile_read(ckks_ctx* ctx, uint32_t index, const char** name, uint64_t* launches, double* total_ms,
                      uint64_t* alg_bytes);

#ifdef __cplusplus
}
#endif
#endif /* CKKS_MI355X_H */
