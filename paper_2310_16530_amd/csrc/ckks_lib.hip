// Host side of the C ABI declared in include/ckks_mi355x.h: context creation (table
// generation on the host, one upload), argument validation, workspace carving and kernel
// launches.  No device memory is allocated here.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/ckks_mi355x.h"
#include "poly_kernels.h"

typedef unsigned __int128 u128;

// ------------------------------------------------------------------ host modular helpers
static inline u64 h_mulmod(u64 a, u64 b, u64 m) { return (u64)(((u128)a * b) % m); }
static u64 h_powmod(u64 b, u64 e, u64 m) {
    u64 r = 1 % m;
    b %= m;
    while (e) {
        if (e & 1) r = h_mulmod(r, b, m);
        b = h_mulmod(b, b, m);
        e >>= 1;
    }
    return r;
}
static inline u64 h_invmod(u64 a, u64 m) { return h_powmod(a % m, m - 2, m); }
static inline u64 h_shoup(u64 w, u64 m) { return (u64)(((u128)w << 64) / m); }
static inline u64 h_mont(u64 w, u64 m) { return (u64)(((u128)w << 64) % m); }
static inline ShoupConst h_sc(u64 w, u64 m) { return ShoupConst{w, h_shoup(w, m)}; }
static u64 h_neg_inv64(u64 q) {  // -q^-1 mod 2^64 by Newton iteration
    u64 x = q;                    // correct to 3 bits (q odd)
    for (int i = 0; i < 6; i++) x *= 2 - q * x;
    return (u64)0 - x;
}
static u32 h_bitrev(u32 x, u32 bits) {
    u32 r = 0;
    for (u32 i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}
static bool h_is_prime(u64 n) {
    if (n < 2) return false;
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 p : bases) {
        if (n % p == 0) return n == p;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) {
        d >>= 1;
        r++;
    }
    for (u64 a : bases) {
        u64 x = h_powmod(a, d, n);
        if (x == 1 || x == n - 1) continue;
        bool comp = true;
        for (int i = 1; i < r; i++) {
            x = h_mulmod(x, x, n);
            if (x == n - 1) {
                comp = false;
                break;
            }
        }
        if (comp) return false;
    }
    return true;
}
// smallest primitive 2N-th root of unity: minimum over the odd powers of any one of them
static u64 h_min_root(u64 m, u32 logN) {
    const u64 N = 1ull << logN;
    u64 root = 0;
    for (u64 x = 2; x < m && !root; x++) {
        u64 y = h_powmod(x, (m - 1) / (2 * N), m);
        if (h_powmod(y, N, m) == m - 1) root = y;
    }
    u64 sq = h_mulmod(root, root, m), cur = root, best = root;
    for (u64 k = 1; k < N; k++) {
        cur = h_mulmod(cur, sq, m);
        if (cur < best) best = cur;
    }
    return best;
}

// ------------------------------------------------------------------------------ context
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct TableLayout {
    size_t tw, pc, up_hatinv, up_chat, dn_hatinv, dn_chat, pinv, total;
};

static TableLayout table_layout(u32 logN, u32 L, u32 K) {
    const size_t N = (size_t)1 << logN, D = L + K;
    TableLayout t;
    size_t o = 0;
    t.tw = o;
    o += align256(D * 4 * N * sizeof(u64));
    t.pc = o;
    o += align256(D * sizeof(PrimeConst));
    t.up_hatinv = o;
    o += align256(L * sizeof(ShoupConst));
    t.up_chat = o;
    o += align256(L * D * sizeof(u64));
    t.dn_hatinv = o;
    o += align256((K ? K : 1) * sizeof(ShoupConst));
    t.dn_chat = o;
    o += align256((K ? K : 1) * L * sizeof(u64));
    t.pinv = o;
    o += align256(L * sizeof(ShoupConst));
    t.total = o;
    return t;
}

// per-kernel timing: when enabled, every launch is bracketed by two HIP events recorded on the
// launch stream; ckks_profile_read waits for them and sums elapsed time per kernel.
enum ProfKind {
    PK_NTT_FWD_STRIDED = 0, PK_NTT_FWD_CONTIG, PK_NTT_INV_CONTIG, PK_NTT_INV_STRIDED, PK_MODUP, PK_MODDOWN,
    PK_INNER, PK_PREP, PK_FINAL, PK_AUTOMORPH, PK_COUNT
};
static const char* const prof_names[PK_COUNT] = {
    "ntt_fwd_strided_kernel", "ntt_fwd_contig_kernel", "ntt_inv_contig_kernel", "ntt_inv_strided_kernel",
    "modup_kernel", "moddown_kernel", "inner_product_kernel", "prep_kernel", "final_kernel", "automorph_kernel"};
static_assert(PK_COUNT == CKKS_PROF_KINDS, "header and library disagree on the number of kernel kinds");

struct ProfRec {
    int kind;
    hipEvent_t a, b;
};
struct ProfState {
    bool on = false;
    std::vector<ProfRec> pending;
    std::vector<hipEvent_t> pool;
    double ms[PK_COUNT] = {0};
    u64 launches[PK_COUNT] = {0}, bytes[PK_COUNT] = {0};
};

struct ckks_ctx {
    u32 logN, L, K, dnum, alpha, D;
    std::vector<u64> primes, psi;
    NttTables ntt;
    ConvTables conv;
    mutable std::string err;
    mutable ProfState prof;
};

static hipEvent_t prof_event(ProfState& p) {
    if (!p.pool.empty()) {
        hipEvent_t e = p.pool.back();
        p.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct ProfScope {
    ProfState* p = nullptr;
    hipStream_t s;
    ProfRec rec;
    ProfScope(const ckks_ctx* c, int kind, u64 alg_bytes, hipStream_t stream) : s(stream) {
        if (!c->prof.on) return;
        p = &c->prof;
        p->launches[kind]++;
        p->bytes[kind] += alg_bytes;
        rec.kind = kind;
        rec.a = prof_event(*p);
        rec.b = prof_event(*p);
        if (!rec.a || !rec.b) {
            p = nullptr;
            return;
        }
        (void)hipEventRecord(rec.a, s);
    }
    ~ProfScope() {
        if (!p) return;
        (void)hipEventRecord(rec.b, s);
        p->pending.push_back(rec);
    }
};

static int fail(const ckks_ctx* c, int code, const char* msg) {
    if (c) c->err = msg;
    return code;
}

static int check_shape(u32 logN, u32 L, u32 K, u32 dnum) {
    if (logN < CKKS_MIN_LOGN || logN > CKKS_MAX_LOGN) return CKKS_EUNSUPPORTED;
    if (L == 0 || dnum == 0) return CKKS_EINVAL;
    if (L + K > CKKS_MAX_PRIMES) return CKKS_EUNSUPPORTED;
    if (L % dnum) return CKKS_EUNSUPPORTED;
    if (K > CKKS_MAX_DIGIT) return CKKS_EUNSUPPORTED;
    if (K > 0 && L / dnum > CKKS_MAX_DIGIT) return CKKS_EUNSUPPORTED;
    return CKKS_OK;
}

extern "C" int ckks_table_bytes(uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, size_t* bytes) {
    if (!bytes) return CKKS_EINVAL;
    int rc = check_shape(logN, L, K, dnum);
    if (rc) return rc;
    *bytes = table_layout(logN, L, K).total;
    return CKKS_OK;
}

extern "C" int ckks_ctx_create(ckks_ctx** out, uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum,
                               const uint64_t* h_primes, const uint64_t* h_psi, void* d_tables, size_t table_bytes,
                               void* stream) {
    if (!out) return CKKS_EINVAL;
    *out = nullptr;
    if (!h_primes || !d_tables) return CKKS_EINVAL;
    int rc = check_shape(logN, L, K, dnum);
    if (rc) return rc;
    if (((uintptr_t)d_tables) & 255) return CKKS_EINVAL;
    const TableLayout lay = table_layout(logN, L, K);
    if (table_bytes < lay.total) return CKKS_ENOMEM;
    const u32 D = L + K, alpha = L / dnum;
    const size_t N = (size_t)1 << logN;
    for (u32 i = 0; i < D; i++) {
        const u64 m = h_primes[i];
        if (m >> CKKS_MAX_PRIME_BITS) return CKKS_EUNSUPPORTED;
        if (m < 2 * N || (m - 1) % (2 * N) != 0) return CKKS_EINVAL;
        if (!h_is_prime(m)) return CKKS_EINVAL;
        for (u32 k = 0; k < i; k++)
            if (h_primes[k] == m) return CKKS_EINVAL;
        if (h_psi && h_powmod(h_psi[i], N, m) != m - 1) return CKKS_EINVAL;
    }

    ckks_ctx* c = new ckks_ctx();
    c->logN = logN, c->L = L, c->K = K, c->dnum = dnum, c->alpha = alpha, c->D = D;
    c->primes.assign(h_primes, h_primes + D);
    c->psi.resize(D);

    std::vector<unsigned char> host(lay.total, 0);
    u64* tw = (u64*)(host.data() + lay.tw);
    PrimeConst* pc = (PrimeConst*)(host.data() + lay.pc);
    std::vector<u64> pw(N);
    for (u32 i = 0; i < D; i++) {
        const u64 m = c->primes[i];
        const u64 psi = h_psi ? h_psi[i] : h_min_root(m, logN);
        c->psi[i] = psi;
        const u64 psi_inv = h_invmod(psi, m);
        u64* fw = tw + (size_t)i * 4 * N;
        for (int dir = 0; dir < 2; dir++) {
            const u64 base = dir ? psi_inv : psi;
            pw[0] = 1;
            for (size_t e = 1; e < N; e++) pw[e] = h_mulmod(pw[e - 1], base, m);
            u64* w = fw + (size_t)dir * 2 * N;
            for (size_t k = 0; k < N; k++) {
                w[k] = pw[h_bitrev((u32)k, logN)];
                w[N + k] = h_shoup(w[k], m);
            }
        }
        PrimeConst& p = pc[i];
        p.q = m;
        p.qneg = h_neg_inv64(m);
        p.r2 = (u64)((((u128)1 << 64) % m) * (((u128)1 << 64) % m) % m);
        p.ninv = h_invmod(N % m, m);
        p.ninv_p = h_shoup(p.ninv, m);
        p.wlast = h_mulmod(fw[2 * N + 1], p.ninv, m);
        p.wlast_p = h_shoup(p.wlast, m);
        p.pad = 0;
    }
    // ModUp constants per digit
    ShoupConst* up_hatinv = (ShoupConst*)(host.data() + lay.up_hatinv);
    u64* up_chat = (u64*)(host.data() + lay.up_chat);
    for (u32 j = 0; j < dnum; j++) {
        for (u32 ii = 0; ii < alpha; ii++) {
            const u32 i = j * alpha + ii;
            const u64 qi = c->primes[i];
            u64 hat = 1;
            for (u32 kk = 0; kk < alpha; kk++)
                if (kk != ii) hat = h_mulmod(hat, c->primes[j * alpha + kk] % qi, qi);
            up_hatinv[i] = h_sc(h_invmod(hat, qi), qi);
            for (u32 t = 0; t < D; t++) {
                if (t >= j * alpha && t < (j + 1) * alpha) continue;
                const u64 mt = c->primes[t];
                u64 hb = 1;
                for (u32 kk = 0; kk < alpha; kk++)
                    if (kk != ii) hb = h_mulmod(hb, c->primes[j * alpha + kk] % mt, mt);
                up_chat[(size_t)i * D + t] = h_mont(hb, mt);
            }
        }
    }
    // ModDown constants
    ShoupConst* dn_hatinv = (ShoupConst*)(host.data() + lay.dn_hatinv);
    u64* dn_chat = (u64*)(host.data() + lay.dn_chat);
    ShoupConst* pinv = (ShoupConst*)(host.data() + lay.pinv);
    for (u32 k = 0; k < K; k++) {
        const u64 pk = c->primes[L + k];
        u64 hat = 1;
        for (u32 kk = 0; kk < K; kk++)
            if (kk != k) hat = h_mulmod(hat, c->primes[L + kk] % pk, pk);
        dn_hatinv[k] = h_sc(h_invmod(hat, pk), pk);
        for (u32 i = 0; i < L; i++) {
            const u64 qi = c->primes[i];
            u64 hb = 1;
            for (u32 kk = 0; kk < K; kk++)
                if (kk != k) hb = h_mulmod(hb, c->primes[L + kk] % qi, qi);
            dn_chat[(size_t)k * L + i] = h_mont(hb, qi);
        }
    }
    for (u32 i = 0; i < L; i++) {
        const u64 qi = c->primes[i];
        u64 P = 1;
        for (u32 k = 0; k < K; k++) P = h_mulmod(P, c->primes[L + k] % qi, qi);
        pinv[i] = h_sc(h_invmod(P, qi), qi);
    }

    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(d_tables, host.data(), lay.total, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        delete c;
        return CKKS_EHIP;
    }
    unsigned char* dbase = (unsigned char*)d_tables;
    c->ntt.tw = (const u64*)(dbase + lay.tw);
    c->ntt.pc = (const PrimeConst*)(dbase + lay.pc);
    c->ntt.logN = logN;
    c->conv.pc = c->ntt.pc;
    c->conv.up_hatinv = (const ShoupConst*)(dbase + lay.up_hatinv);
    c->conv.up_chat = (const u64*)(dbase + lay.up_chat);
    c->conv.dn_hatinv = (const ShoupConst*)(dbase + lay.dn_hatinv);
    c->conv.dn_chat = (const u64*)(dbase + lay.dn_chat);
    c->conv.pinv = (const ShoupConst*)(dbase + lay.pinv);
    *out = c;
    return CKKS_OK;
}

static void prof_drain(ProfState& p) {
    for (ProfRec& r : p.pending) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) p.ms[r.kind] += ms;
        p.pool.push_back(r.a);
        p.pool.push_back(r.b);
    }
    p.pending.clear();
}

extern "C" void ckks_ctx_destroy(ckks_ctx* ctx) {
    if (!ctx) return;
    prof_drain(ctx->prof);
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
    delete ctx;
}

extern "C" int ckks_profile_enable(ckks_ctx* ctx, int on) {
    if (!ctx) return CKKS_EINVAL;
    prof_drain(ctx->prof);
    ctx->prof.on = on != 0;
    for (int k = 0; k < PK_COUNT; k++) ctx->prof.ms[k] = 0, ctx->prof.launches[k] = 0, ctx->prof.bytes[k] = 0;
    return CKKS_OK;
}

extern "C" int ckks_profile_read(ckks_ctx* ctx, uint32_t kind, const char** name, uint64_t* launches,
                                 double* total_ms, uint64_t* alg_bytes) {
    if (!ctx || kind >= PK_COUNT) return CKKS_EINVAL;
    prof_drain(ctx->prof);
    if (name) *name = prof_names[kind];
    if (launches) *launches = ctx->prof.launches[kind];
    if (total_ms) *total_ms = ctx->prof.ms[kind];
    if (alg_bytes) *alg_bytes = ctx->prof.bytes[kind];
    return CKKS_OK;
}

extern "C" const char* ckks_last_error(const ckks_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

extern "C" uint64_t ckks_ctx_psi(const ckks_ctx* ctx, uint32_t i) { return (ctx && i < ctx->D) ? ctx->psi[i] : 0; }

// ----------------------------------------------------------------------------- launches
static inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

static int hip_check(const ckks_ctx* c, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        c->err = std::string(what) + ": " + hipGetErrorString(e);
        return CKKS_EHIP;
    }
    return CKKS_OK;
}

template <int A>
static void launch_ntt_a(const ckks_ctx* c, u64* data, const LimbMap& map, u32 jobs, bool inverse, hipStream_t s) {
    const u32 tiles = (1u << A) / 16;
    const dim3 grid(jobs * tiles), block(256);
    const u64 bytes = (u64)jobs * 2 * sizeof(u64) << c->logN;  // every limb read once and written once
    if (!inverse) {
        {
            ProfScope ps(c, PK_NTT_FWD_STRIDED, bytes, s);
            hipLaunchKernelGGL(ntt_fwd_strided_kernel<A>, grid, block, 0, s, data, map, c->ntt);
        }
        {
            ProfScope ps(c, PK_NTT_FWD_CONTIG, bytes, s);
            hipLaunchKernelGGL(ntt_fwd_contig_kernel<A>, grid, block, 0, s, data, map, c->ntt);
        }
    } else {
        {
            ProfScope ps(c, PK_NTT_INV_CONTIG, bytes, s);
            hipLaunchKernelGGL(ntt_inv_contig_kernel<A>, grid, block, 0, s, data, map, c->ntt);
        }
        {
            ProfScope ps(c, PK_NTT_INV_STRIDED, bytes, s);
            hipLaunchKernelGGL(ntt_inv_strided_kernel<A>, grid, block, 0, s, data, map, c->ntt);
        }
    }
}

// jobs = number of limbs the map enumerates
static void launch_ntt(const ckks_ctx* c, u64* data, const LimbMap& map, u32 jobs, bool inverse, hipStream_t s) {
    if (jobs == 0) return;
    switch (c->logN - 8) {
        case 4: launch_ntt_a<4>(c, data, map, jobs, inverse, s); break;
        case 5: launch_ntt_a<5>(c, data, map, jobs, inverse, s); break;
        case 6: launch_ntt_a<6>(c, data, map, jobs, inverse, s); break;
        case 7: launch_ntt_a<7>(c, data, map, jobs, inverse, s); break;
        case 8: launch_ntt_a<8>(c, data, map, jobs, inverse, s); break;
    }
}

static LimbMap plain_map(u32 n_limbs, u32 prime_first) { return LimbMap{n_limbs, n_limbs, 0, prime_first, 0, 1}; }

template <int AL>
static void launch_modup_a(const ckks_ctx* c, const u64* in, u64* out, u32 batch, int write_own, hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, c->dnum, batch), block(256);
    const u64 limbs = (u64)batch * (c->L + (u64)c->dnum * (c->D - c->alpha) + (write_own ? c->L : 0));
    ProfScope ps(c, PK_MODUP, limbs * sizeof(u64) << c->logN, s);
    hipLaunchKernelGGL(modup_kernel<AL>, grid, block, 0, s, in, out, c->conv, c->logN, c->L, c->D, c->dnum, write_own);
}
static void launch_modup(const ckks_ctx* c, const u64* in, u64* out, u32 batch, int write_own, hipStream_t s) {
    switch (c->alpha) {
        case 1: launch_modup_a<1>(c, in, out, batch, write_own, s); break;
        case 2: launch_modup_a<2>(c, in, out, batch, write_own, s); break;
        case 3: launch_modup_a<3>(c, in, out, batch, write_own, s); break;
        case 4: launch_modup_a<4>(c, in, out, batch, write_own, s); break;
        case 5: launch_modup_a<5>(c, in, out, batch, write_own, s); break;
        case 6: launch_modup_a<6>(c, in, out, batch, write_own, s); break;
        case 7: launch_modup_a<7>(c, in, out, batch, write_own, s); break;
        case 8: launch_modup_a<8>(c, in, out, batch, write_own, s); break;
    }
}

template <int KK, bool FUSE>
static void launch_moddown_k(const ckks_ctx* c, const u64* in, u64* out, u32 groups, hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, groups), block(256);
    const u64 limbs = (u64)groups * (c->K + c->L + (FUSE ? c->L : 0));
    ProfScope ps(c, PK_MODDOWN, limbs * sizeof(u64) << c->logN, s);
    hipLaunchKernelGGL((moddown_kernel<KK, FUSE>), grid, block, 0, s, in, out, c->conv, c->logN, c->L, c->D);
}
template <bool FUSE>
static void launch_moddown(const ckks_ctx* c, const u64* in, u64* out, u32 groups, hipStream_t s) {
    switch (c->K) {
        case 1: launch_moddown_k<1, FUSE>(c, in, out, groups, s); break;
        case 2: launch_moddown_k<2, FUSE>(c, in, out, groups, s); break;
        case 3: launch_moddown_k<3, FUSE>(c, in, out, groups, s); break;
        case 4: launch_moddown_k<4, FUSE>(c, in, out, groups, s); break;
        case 5: launch_moddown_k<5, FUSE>(c, in, out, groups, s); break;
        case 6: launch_moddown_k<6, FUSE>(c, in, out, groups, s); break;
        case 7: launch_moddown_k<7, FUSE>(c, in, out, groups, s); break;
        case 8: launch_moddown_k<8, FUSE>(c, in, out, groups, s); break;
    }
}

// ---------------------------------------------------------------------- workspace carving
struct Workspace {
    u64 *x, *dt, *cp, *cv;
};

static size_t ks_workspace_words(const ckks_ctx* c, u32 x_groups, u32 dt_groups, u32 cp_groups) {
    const size_t N = (size_t)1 << c->logN;
    return ((size_t)x_groups * c->L + (size_t)dt_groups * c->dnum * c->D + (size_t)cp_groups * 2 * c->D +
            (size_t)cp_groups * 2 * c->L) * N;
}

static Workspace carve(const ckks_ctx* c, void* ws, u32 x_groups, u32 dt_groups, u32 cp_groups) {
    const size_t N = (size_t)1 << c->logN;
    Workspace w;
    w.x = (u64*)ws;
    w.dt = w.x + (size_t)x_groups * c->L * N;
    w.cp = w.dt + (size_t)dt_groups * c->dnum * c->D * N;
    w.cv = w.cp + (size_t)cp_groups * 2 * c->D * N;
    return w;
}

extern "C" int ckks_workspace_bytes(const ckks_ctx* ctx, int op, uint32_t batch_or_nrot, size_t* bytes) {
    if (!ctx || !bytes) return CKKS_EINVAL;
    if (batch_or_nrot == 0) return fail(ctx, CKKS_EINVAL, "batch must be positive");
    switch (op) {
        case CKKS_OP_NTT:
        case CKKS_OP_MODUP:
        case CKKS_OP_MODDOWN:
        case CKKS_OP_AUTOMORPH: *bytes = 0; return CKKS_OK;
        case CKKS_OP_KEYSWITCH:
        case CKKS_OP_HMULT_RELIN:
        case CKKS_OP_HROT:
            if (ctx->K == 0) return fail(ctx, CKKS_EUNSUPPORTED, "context has no special primes");
            *bytes = ks_workspace_words(ctx, batch_or_nrot, batch_or_nrot, batch_or_nrot) * sizeof(u64);
            return CKKS_OK;
        case CKKS_OP_HROT_HOISTED_MAC: {
            if (ctx->K == 0) return fail(ctx, CKKS_EUNSUPPORTED, "context has no special primes");
            const u32 chunk = batch_or_nrot < CKKS_ROT_CHUNK ? batch_or_nrot : CKKS_ROT_CHUNK;
            *bytes = ks_workspace_words(ctx, 1, 1, chunk) * sizeof(u64);
            return CKKS_OK;
        }
    }
    return fail(ctx, CKKS_EINVAL, "unknown op selector");
}

// --------------------------------------------------------------------------- entry points
static int check_limb_range(const ckks_ctx* c, u32 prime_first, u32 n_limbs, u32 batch) {
    if (n_limbs == 0 || batch == 0) return fail(c, CKKS_EINVAL, "n_limbs and batch must be positive");
    if ((u64)prime_first + n_limbs > c->D) return fail(c, CKKS_EINVAL, "limb range exceeds the prime chain");
    if ((u64)n_limbs * batch > (1u << 20)) return fail(c, CKKS_EINVAL, "batch too large");
    return CKKS_OK;
}

static int ntt_entry(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                     void* stream, bool inverse) {
    if (!ctx) return CKKS_EINVAL;
    if (!d_x || misaligned(d_x, 16)) return fail(ctx, CKKS_EINVAL, "d_x is null or not 16-byte aligned");
    int rc = check_limb_range(ctx, prime_first, n_limbs, batch);
    if (rc) return rc;
    launch_ntt(ctx, d_x, plain_map(n_limbs, prime_first), n_limbs * batch, inverse, (hipStream_t)stream);
    return hip_check(ctx, inverse ? "ckks_intt" : "ckks_ntt");
}

extern "C" int ckks_ntt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                        void* stream) {
    return ntt_entry(ctx, d_x, prime_first, n_limbs, batch, stream, false);
}

extern "C" int ckks_intt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                         void* stream) {
    return ntt_entry(ctx, d_x, prime_first, n_limbs, batch, stream, true);
}

static int check_ks_ctx(const ckks_ctx* c, u32 batch) {
    if (c->K == 0) return fail(c, CKKS_EUNSUPPORTED, "context has no special primes");
    if (batch == 0 || batch > 4096) return fail(c, CKKS_EINVAL, "batch out of range");
    return CKKS_OK;
}

extern "C" int ckks_modup(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(ctx, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(ctx, batch);
    if (rc) return rc;
    launch_modup(ctx, d_in, d_out, batch, 1, (hipStream_t)stream);
    return hip_check(ctx, "ckks_modup");
}

extern "C" int ckks_moddown(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(ctx, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(ctx, batch);
    if (rc) return rc;
    launch_moddown<true>(ctx, d_in, d_out, batch, (hipStream_t)stream);
    return hip_check(ctx, "ckks_moddown");
}

static int check_galois(const ckks_ctx* c, u32 g) {
    if ((g & 1) == 0 || g >= (2u << c->logN)) return fail(c, CKKS_EINVAL, "Galois element must be odd and below 2N");
    return CKKS_OK;
}

extern "C" int ckks_automorph(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t prime_first,
                              uint32_t n_limbs, uint32_t galois, int eval_domain, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(ctx, CKKS_EINVAL, "null or misaligned buffer");
    if (d_in == d_out) return fail(ctx, CKKS_EINVAL, "automorphism cannot run in place");
    int rc = check_limb_range(ctx, prime_first, n_limbs, batch);
    if (rc) return rc;
    rc = check_galois(ctx, galois);
    if (rc) return rc;
    if (batch > 65535) return fail(ctx, CKKS_EINVAL, "batch too large");
    const dim3 grid((1u << ctx->logN) / 256, n_limbs, batch), block(256);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(ctx, PK_AUTOMORPH, (u64)batch * n_limbs * 2 * sizeof(u64) << ctx->logN, s);
    if (eval_domain) {
        hipLaunchKernelGGL(automorph_eval_kernel, grid, block, 0, s, d_in, d_out, ctx->logN, n_limbs, galois);
    } else {
        // inverse of g modulo 2N (a power of two): Newton iteration on 32-bit words, then mask
        u32 inv = galois;
        for (int i = 0; i < 5; i++) inv *= 2 - galois * inv;
        inv &= (2u << ctx->logN) - 1;
        hipLaunchKernelGGL(automorph_coeff_kernel, grid, block, 0, s, d_in, d_out, ctx->ntt.pc, ctx->logN, n_limbs,
                           prime_first, inv);
    }
    return hip_check(ctx, "ckks_automorph");
}

// Shared tail of every key switch.  On entry w.x holds the evaluation-form polynomial(s) to
// switch, [x_groups][L][N], and the own-digit limbs of w.dt already hold the same values.
// Leaves c' in w.cp ([cp_groups][2][D][N]) and NTT(Conv_{P->Q}(INTT(c'|P))) in w.cv.
static void decompose_extend(const ckks_ctx* c, const Workspace& w, u32 groups, hipStream_t s) {
    launch_ntt(c, w.x, plain_map(c->L, 0), groups * c->L, true, s);
    launch_modup(c, w.x, w.dt, groups, 0, s);
    const LimbMap ext = {c->D - c->alpha, c->D, 0, 0, c->alpha, c->dnum};
    launch_ntt(c, w.dt, ext, groups * c->dnum * (c->D - c->alpha), false, s);
}

static void moddown_tail(const ckks_ctx* c, const Workspace& w, u32 cp_groups, hipStream_t s) {
    const LimbMap special = {c->K, c->D, c->L, 0, 0, 1};
    launch_ntt(c, w.cp, special, cp_groups * 2 * c->K, true, s);
    launch_moddown<false>(c, w.cp, w.cv, cp_groups * 2, s);
    launch_ntt(c, w.cv, plain_map(c->L, 0), cp_groups * 2 * c->L, false, s);
}

static int check_ks_args(const ckks_ctx* c, const void* a, const void* b, const void* out, u32 batch, int op,
                         const void* ws, size_t ws_bytes) {
    if (!a || !b || !out || misaligned(a, 16) || misaligned(b, 16) || misaligned(out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(c, batch);
    if (rc) return rc;
    if (!ws || misaligned(ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    rc = ckks_workspace_bytes(c, op, batch, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(c, CKKS_ENOMEM, "workspace too small");
    return CKKS_OK;
}

template <int MODE>
static void launch_prep(const ckks_ctx* c, const u64* in1, const u64* in2, const Workspace& w, u32 batch, u32 galois,
                        hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, c->L, batch), block(256);
    const u64 limbs = (u64)batch * c->L * (MODE == PREP_TENSOR_D2 ? 4 : 3);
    ProfScope ps(c, PK_PREP, limbs * sizeof(u64) << c->logN, s);
    hipLaunchKernelGGL(prep_kernel<MODE>, grid, block, 0, s, in1, in2, w.x, w.dt, c->ntt.pc, c->logN, c->L, c->D,
                       c->dnum, c->alpha, galois);
}

static void launch_inner_shared_key(const ckks_ctx* c, const Workspace& w, const u64* key, u32 batch, hipStream_t s) {
    const size_t N = (size_t)1 << c->logN;
    KeyPtrs kp;
    memset(&kp, 0, sizeof(kp));
    kp.key[0] = key;
    const dim3 grid((1u << c->logN) / 256, c->D, batch), block(256);
    // extended digits read, c' written, the shared key read once
    const u64 limbs = (u64)batch * (c->dnum + 2) * c->D + (u64)c->dnum * 2 * c->D;
    ProfScope ps(c, PK_INNER, limbs * sizeof(u64) << c->logN, s);
    hipLaunchKernelGGL(inner_product_kernel<false>, grid, block, 0, s, (const u64*)w.dt, (size_t)c->dnum * c->D * N, kp,
                       w.cp, c->ntt.pc, c->logN, c->D, c->dnum);
}

template <int MODE>
static void launch_final(const ckks_ctx* c, const FinalArgs& fa, u32 groups, hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, c->L, MODE == FIN_HOISTED ? 2 : groups * 2), block(256);
    u64 limbs;  // c' and conv read, output written, plus the mode's extra operands
    if (MODE == FIN_HOISTED) limbs = (u64)fa.n_rot * c->L * (4 + 1 + 1) + (u64)c->L * (2 + (fa.accumulate ? 2 : 0));
    else limbs = (u64)groups * c->L * (6 + (MODE == FIN_HMULT ? 4 : MODE == FIN_HROT ? 1 : 0));
    ProfScope ps(c, PK_FINAL, limbs * sizeof(u64) << c->logN, s);
    hipLaunchKernelGGL(final_kernel<MODE>, grid, block, 0, s, fa, c->conv, c->logN, c->L, c->D);
}

extern "C" int ckks_keyswitch(ckks_ctx* ctx, const uint64_t* d_d, const uint64_t* d_key, uint64_t* d_out,
                              uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    int rc = check_ks_args(ctx, d_d, d_key, d_out, batch, CKKS_OP_KEYSWITCH, d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(ctx, d_ws, batch, batch, batch);
    launch_prep<PREP_COPY>(ctx, d_d, nullptr, w, batch, 1, s);
    decompose_extend(ctx, w, batch, s);
    launch_inner_shared_key(ctx, w, d_key, batch, s);
    moddown_tail(ctx, w, batch, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cp = w.cp, fa.cv = w.cv, fa.out = d_out;
    launch_final<FIN_KS>(ctx, fa, batch, s);
    return hip_check(ctx, "ckks_keyswitch");
}

extern "C" int ckks_hmult_relin(ckks_ctx* ctx, const uint64_t* d_ct1, const uint64_t* d_ct2, const uint64_t* d_evk,
                                uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    if (!d_ct2 || misaligned(d_ct2, 16)) return fail(ctx, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_args(ctx, d_ct1, d_evk, d_out, batch, CKKS_OP_HMULT_RELIN, d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(ctx, d_ws, batch, batch, batch);
    launch_prep<PREP_TENSOR_D2>(ctx, d_ct1, d_ct2, w, batch, 1, s);
    decompose_extend(ctx, w, batch, s);
    launch_inner_shared_key(ctx, w, d_evk, batch, s);
    moddown_tail(ctx, w, batch, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cp = w.cp, fa.cv = w.cv, fa.out = d_out, fa.ct1 = d_ct1, fa.ct2 = d_ct2;
    launch_final<FIN_HMULT>(ctx, fa, batch, s);
    return hip_check(ctx, "ckks_hmult_relin");
}

extern "C" int ckks_hrot(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t galois, const uint64_t* d_rk, uint64_t* d_out,
                         uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    int rc = check_ks_args(ctx, d_ct, d_rk, d_out, batch, CKKS_OP_HROT, d_ws, ws_bytes);
    if (rc) return rc;
    rc = check_galois(ctx, galois);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(ctx, d_ws, batch, batch, batch);
    launch_prep<PREP_ROT_A>(ctx, d_ct, nullptr, w, batch, galois, s);
    decompose_extend(ctx, w, batch, s);
    launch_inner_shared_key(ctx, w, d_rk, batch, s);
    moddown_tail(ctx, w, batch, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cp = w.cp, fa.cv = w.cv, fa.out = d_out, fa.ct1 = d_ct, fa.galois[0] = galois;
    launch_final<FIN_HROT>(ctx, fa, batch, s);
    return hip_check(ctx, "ckks_hrot");
}

extern "C" int ckks_hrot_hoisted_mac(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                                     const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out,
                                     void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    if (!h_galois || !h_rk_ptrs) return fail(ctx, CKKS_EINVAL, "null host array");
    if (n_rot == 0 || n_rot > 65535) return fail(ctx, CKKS_EINVAL, "n_rot out of range");
    if (!d_ct || !d_pt || !d_out || misaligned(d_ct, 16) || misaligned(d_pt, 16) || misaligned(d_out, 16))
        return fail(ctx, CKKS_EINVAL, "null or misaligned buffer");
    if (!d_ws || misaligned(d_ws, 256)) return fail(ctx, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    int rc = ckks_workspace_bytes(ctx, CKKS_OP_HROT_HOISTED_MAC, n_rot, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(ctx, CKKS_ENOMEM, "workspace too small");
    for (u32 r = 0; r < n_rot; r++) {
        if (!h_rk_ptrs[r] || misaligned(h_rk_ptrs[r], 16)) return fail(ctx, CKKS_EINVAL, "null or misaligned key");
        rc = check_galois(ctx, h_galois[r]);
        if (rc) return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    const size_t N = (size_t)1 << ctx->logN;
    const u32 chunk_max = n_rot < CKKS_ROT_CHUNK ? n_rot : CKKS_ROT_CHUNK;
    const Workspace w = carve(ctx, d_ws, 1, 1, chunk_max);
    // hoisted part: decompose a = ct[1] once
    {
        const dim3 grid((1u << ctx->logN) / 256, ctx->L, 1), block(256);
        ProfScope ps(ctx, PK_PREP, (u64)ctx->L * 3 * sizeof(u64) << ctx->logN, s);
        hipLaunchKernelGGL(prep_kernel<PREP_COPY>, grid, block, 0, s, d_ct + (size_t)ctx->L * N, (const u64*)nullptr,
                           w.x, w.dt, ctx->ntt.pc, ctx->logN, ctx->L, ctx->D, ctx->dnum, ctx->alpha, 1u);
    }
    decompose_extend(ctx, w, 1, s);
    for (u32 r0 = 0; r0 < n_rot; r0 += CKKS_ROT_CHUNK) {
        const u32 nr = (n_rot - r0) < CKKS_ROT_CHUNK ? (n_rot - r0) : CKKS_ROT_CHUNK;
        KeyPtrs kp;
        memset(&kp, 0, sizeof(kp));
        FinalArgs fa;
        memset(&fa, 0, sizeof(fa));
        for (u32 r = 0; r < nr; r++) {
            kp.key[r] = h_rk_ptrs[r0 + r];
            kp.galois[r] = h_galois[r0 + r];
            fa.galois[r] = h_galois[r0 + r];
        }
        const dim3 grid((1u << ctx->logN) / 256, ctx->D, nr), block(256);
        {
            // per rotation: the shared extended digits gathered, its key read, c' written
            const u64 limbs = (u64)nr * ((u64)ctx->dnum * ctx->D + (u64)ctx->dnum * 2 * ctx->D + 2 * ctx->D);
            ProfScope ps(ctx, PK_INNER, limbs * sizeof(u64) << ctx->logN, s);
            hipLaunchKernelGGL(inner_product_kernel<true>, grid, block, 0, s, (const u64*)w.dt, (size_t)0, kp, w.cp,
                               ctx->ntt.pc, ctx->logN, ctx->D, ctx->dnum);
        }
        moddown_tail(ctx, w, nr, s);
        fa.cp = w.cp, fa.cv = w.cv, fa.out = d_out, fa.ct1 = d_ct, fa.pt = d_pt + (size_t)r0 * ctx->L * N;
        fa.n_rot = nr, fa.accumulate = r0 ? 1 : 0;
        launch_final<FIN_HOISTED>(ctx, fa, 1, s);
    }
    return hip_check(ctx, "ckks_hrot_hoisted_mac");
}
