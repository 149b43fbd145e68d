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
#include "kernels.h"

typedef unsigned __int128 u128;
static_assert(CKKS_ROT_CHUNK == CKKS_ROTATIONS_PER_LAUNCH, "the public constant must match the kernels' argument arrays");

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

static inline u32 u8_of(u64 z, u32 k) { return (u32)(z >> (8 * k)) & 0xffu; }

// ------------------------------------------------------------------------------ context
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// The caller's table buffer holds one block shared by every level (per-prime twiddles and
// constants over the whole chain), one block of conversion constants per level ell = 1..L (basis
// q_0..q_{ell-1}, p_0..p_{K-1}) and one small block per rescale step ell -> ell-1 (ell = 2..L).
struct SharedLayout {
    size_t tw_int, tw_fp, pc, sc_plain, sc_dn, dn_hatinv, end;
};
struct LevelLayout {
    size_t sc_up, up_hatinv, up_chat, up_chat_fp, up_fp_ok, dn_chat, dn_chat_fp, dn_fp_ok, pinv, pmod, up_tiles, up_aop,
        dn_tiles, dn_aop, end;
};

// Conversion on the matrix cores: targets per tile and the bound on tiles for a basis of `targets` limbs; ks = products
// per coefficient group = ceil(sources / 4), used for 2..8 sources only
// CKKS_MFMA_NTT: targets per lane half of a tile.  2 halves the matrix-core work per output but needs 128 registers
// for the converted words alone and spills (1.1 KB per lane); 1 is what runs.
// CKKS_MFMA_UP: the ModUp conversion (6 sources of 50 bits at the benchmark shape) measured the same on the matrix
// cores as on the FP64 pipe (125 vs 124 us), so only the ModDown direction (60-bit sources: 11 FP64 instructions per
// source and output against 19 in total) uses them by default.
#ifndef CKKS_MFMA_NTT
#define CKKS_MFMA_NTT 1
#endif
#ifndef CKKS_MFMA_UP
#define CKKS_MFMA_UP 0
#endif
static inline u32 mfma_ks(u32 sources) { return (sources >= 2 && sources <= 8) ? (sources + 3) / 4 : 0; }
static inline u32 mfma_ks_up(u32 sources) { return CKKS_MFMA_UP ? mfma_ks(sources) : 0; }
static inline u32 mfma_tile_bound(u32 targets) { return (targets + 2 * CKKS_MFMA_NTT - 1) / (2 * CKKS_MFMA_NTT) + 1; }
struct RescaleLayout {
    size_t sc_dn, dn_chat, dn_chat_fp, dn_fp_ok, pinv, end;
};

struct Taker {
    size_t o;
    size_t take(size_t bytes) {
        size_t at = o;
        o += align256(bytes);
        return at;
    }
};

static SharedLayout shared_layout(u32 logN, u32 L, u32 K) {
    const size_t N = (size_t)1 << logN, D = L + K, K1 = K ? K : 1;
    Taker t{0};
    SharedLayout l;
    l.tw_int = t.take(D * 4 * N * sizeof(u64));
    l.tw_fp = t.take(D * 2 * N * sizeof(double));
    l.pc = t.take(D * sizeof(PrimeConst));
    l.sc_plain = t.take(D * sizeof(InvScale));
    l.sc_dn = t.take(K1 * sizeof(InvScale));
    l.dn_hatinv = t.take(K1 * 2 * sizeof(u64));
    l.end = t.o;
    return l;
}

static LevelLayout level_layout(size_t base, u32 ell, u32 K, u32 alpha) {
    const size_t D = ell + K, K1 = K ? K : 1, beta = (ell + alpha - 1) / alpha;
    Taker t{base};
    LevelLayout l;
    l.sc_up = t.take(ell * sizeof(InvScale));
    l.up_hatinv = t.take(ell * 2 * sizeof(u64));
    l.up_chat = t.take(ell * D * sizeof(u64));
    l.up_chat_fp = t.take(ell * D * sizeof(double));
    l.up_fp_ok = t.take(beta * D * sizeof(u32));
    l.dn_chat = t.take(K1 * ell * sizeof(u64));
    l.dn_chat_fp = t.take(K1 * ell * sizeof(double));
    l.dn_fp_ok = t.take(ell * sizeof(u32));
    l.pinv = t.take(ell * sizeof(PinvConst));
    l.pmod = t.take(ell * sizeof(u64));
    l.up_tiles = t.take((mfma_ks_up(alpha) ? beta * mfma_tile_bound(D) : 0) * sizeof(ConvTile));
    l.up_aop = t.take(beta * mfma_tile_bound(D) * mfma_ks_up(alpha) * 128 * sizeof(u64));
    l.dn_tiles = t.take(mfma_tile_bound(ell) * sizeof(ConvTile));
    l.dn_aop = t.take(mfma_tile_bound(ell) * mfma_ks(K) * 128 * sizeof(u64));
    l.end = t.o;
    return l;
}

// rescale from ell limbs to ell - 1: one source prime (q_{ell-1}), targets q_0..q_{ell-2}
static RescaleLayout rescale_layout(size_t base, u32 ell) {
    const size_t T = ell - 1;
    Taker t{base};
    RescaleLayout l;
    l.sc_dn = t.take(sizeof(InvScale));
    l.dn_chat = t.take(T * sizeof(u64));
    l.dn_chat_fp = t.take(T * sizeof(double));
    l.dn_fp_ok = t.take(T * sizeof(u32));
    l.pinv = t.take(T * sizeof(PinvConst));
    l.end = t.o;
    return l;
}

// ModDown merged with the rescale after it, from level ell: sources q_{ell-1}, p_0..p_{K-1}; targets q_0..q_{ell-2}
struct MergedLayout {
    size_t sc_dn, dn_chat, dn_chat_fp, dn_fp_ok, pinv, dn_tiles, dn_aop, end;
};
static MergedLayout merged_layout(size_t base, u32 ell, u32 K) {
    const size_t T = ell - 1, S = K + 1;
    Taker t{base};
    MergedLayout l;
    l.sc_dn = t.take(S * sizeof(InvScale));
    l.dn_chat = t.take(S * T * sizeof(u64));
    l.dn_chat_fp = t.take(S * T * sizeof(double));
    l.dn_fp_ok = t.take(T * sizeof(u32));
    l.pinv = t.take(T * sizeof(PinvConst));
    l.dn_tiles = t.take(mfma_tile_bound(T) * sizeof(ConvTile));
    l.dn_aop = t.take(mfma_tile_bound(T) * mfma_ks(S) * 128 * sizeof(u64));
    l.end = t.o;
    return l;
}

static size_t table_total(u32 logN, u32 L, u32 K, u32 dnum) {
    size_t o = shared_layout(logN, L, K).end;
    for (u32 ell = 1; ell <= L; ell++) o = level_layout(o, ell, K, (L + dnum - 1) / dnum).end;
    for (u32 ell = 2; ell <= L; ell++) o = rescale_layout(o, ell).end;
    if (K)
        for (u32 ell = 2; ell <= L; ell++) o = merged_layout(o, ell, K).end;
    return o;
}

// per-kernel timing: when enabled, every launch is bracketed by two HIP events recorded on the
// launch stream; ckks_profile_read waits for them and sums elapsed time per kernel instantiation
// (named as the profiler names it, e.g. "fwd_strided_kernel<FpAr, 8, 1>").
struct ProfRec {
    int kind;
    hipEvent_t a, b;
};
struct ProfKindStat {
    std::string name;
    double ms = 0;
    u64 launches = 0, bytes = 0;
};
struct ProfState {
    bool on = false;
    std::vector<ProfRec> pending;
    std::vector<hipEvent_t> pool;
    std::vector<ProfKindStat> kinds;
    int kind_of(const std::string& name) {
        for (size_t i = 0; i < kinds.size(); i++)
            if (kinds[i].name == name) return (int)i;
        kinds.emplace_back();
        kinds.back().name = name;
        return (int)kinds.size() - 1;
    }
};

// Overlap of the two arithmetic classes: between fork() and join() the launches on IntAr limbs
// (integer-VALU bound) go to a side stream and run concurrently with the launches on FpAr limbs
// (memory bound) of the caller's stream.  Ordering is by events only; both streams have default priority.
struct SideStream {
    bool enabled = false;  // off by default; ckks_set_overlap switches it
    bool active = false;
    bool fp_pending = false;  // an FpAr conversion is running on the side stream (see decompose_extend)
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> events;
    size_t next = 0;
};

struct Shared {
    std::string err;
    ProfState prof;
    SideStream side;
};

// One level of the context: everything a launch needs.  `primes` is the level's basis in limb order.
struct View {
    u32 logN = 0, L = 0, K = 0, dnum = 0, alpha = 0, D = 0;
    std::vector<u64> primes;
    Tables tb;
    bool mixed_classes = false;  // both FpAr and IntAr primes present
    Shared* sh = nullptr;
};

// Scratch memory of ckks_rescale_static, the entry point for callers that cannot allocate or bring a
// workspace: one array per GPU, held from the moment the code object is loaded on that GPU until the process
// ends.  In host code the name `scratch` is only a handle for hipGetSymbolAddress: the address a kernel may
// use is looked up once per device (at context creation, with that device current) and kept in the context.
static __device__ __align__(256) unsigned char scratch[CKKS_STATIC_SCRATCH_BYTES];

struct ckks_ctx {
    int device = -1;               // the device that was current at creation: tables and scratch live there
    void* scratch_ptr = nullptr;   // device address of `scratch` on that device
    u32 logN, L, K, dnum, alpha, D;
    std::vector<u64> primes, psi;
    std::vector<View> level;    // [ell], 1 <= ell <= L: key switching at ell active q-limbs; level[L] is the full one
    std::vector<View> rescale;  // [ell], 2 <= ell <= L: the step from ell limbs to ell - 1 (K = 1, "special" prime q_{ell-1})
    std::vector<View> merged;   // [ell], 2 <= ell <= L, K > 0: ModDown from level ell that also divides by q_{ell-1}
    mutable Shared sh;
    const View* full() const { return &level[L]; }
};

static hipEvent_t side_event(SideStream& sd) {
    if (sd.events.size() < 16) {
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        sd.events.push_back(e);
        return e;
    }
    return sd.events[sd.next++ % sd.events.size()];
}

static bool side_stream_ready(SideStream& sd) {
    if (!sd.stream && hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking) != hipSuccess) {
        sd.stream = nullptr;
        sd.enabled = false;
        (void)hipGetLastError();
        return false;
    }
    return true;
}

// From here on IntAr launches go to the side stream, ordered after everything enqueued on s so far.
static void fork_side(const View* c, hipStream_t s) {
    SideStream& sd = c->sh->side;
    if (!sd.enabled || !c->mixed_classes || sd.active) return;
    if (!side_stream_ready(sd)) return;
    hipEvent_t e = side_event(sd);
    if (!e || hipEventRecord(e, s) != hipSuccess || hipStreamWaitEvent(sd.stream, e, 0) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    sd.active = true;
}

// s waits for everything the side stream was given; IntAr launches return to s.
static void join_side(const View* c, hipStream_t s) {
    SideStream& sd = c->sh->side;
    if (!sd.active) return;
    sd.active = false;
    hipEvent_t e = side_event(sd);
    if (!e || hipEventRecord(e, sd.stream) != hipSuccess || hipStreamWaitEvent(s, e, 0) != hipSuccess) {
        // cannot order by event: fall back to a full wait so that correctness never depends on it
        (void)hipGetLastError();
        (void)hipStreamSynchronize(sd.stream);
    }
}

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
    // alg_limbs: limbs (N words each) the launch must read plus write once
    ProfScope(const View* c, const std::string& name, u64 alg_limbs, hipStream_t stream) : s(stream) {
        if (!c->sh->prof.on) return;
        p = &c->sh->prof;
        rec.kind = p->kind_of(name);
        p->kinds[rec.kind].launches++;
        p->kinds[rec.kind].bytes += (alg_limbs * sizeof(u64)) << c->logN;
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

static void prof_drain(ProfState& p) {
    for (ProfRec& r : p.pending) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) p.kinds[r.kind].ms += ms;
        p.pool.push_back(r.a);
        p.pool.push_back(r.b);
    }
    p.pending.clear();
}

static int fail(const ckks_ctx* c, int code, const char* msg) {
    if (c) c->sh.err = msg;
    return code;
}
static int fail(const View* c, int code, const char* msg) {
    if (c) c->sh->err = msg;
    return code;
}

static int check_shape(u32 logN, u32 L, u32 K, u32 dnum) {
    if (logN < CKKS_MIN_LOGN || logN > CKKS_MAX_LOGN) return CKKS_EUNSUPPORTED;
    if (L == 0 || dnum == 0) return CKKS_EINVAL;
    if (L + K > CKKS_MAX_PRIMES) return CKKS_EUNSUPPORTED;
    if (dnum > L) return CKKS_EINVAL;
    const u32 alpha = (L + dnum - 1) / dnum;  // limbs per digit; the last digit is shorter if dnum does not divide L
    if ((L + alpha - 1) / alpha != dnum) return CKKS_EUNSUPPORTED;  // dnum is not the digit count this size gives
    if (K > CKKS_MAX_DIGIT) return CKKS_EUNSUPPORTED;
    if (K > 0 && alpha > CKKS_MAX_DIGIT) return CKKS_EUNSUPPORTED;
    return CKKS_OK;
}

extern "C" int ckks_table_bytes(uint32_t logN, uint32_t L, uint32_t K, uint32_t dnum, size_t* bytes) {
    if (!bytes) return CKKS_EINVAL;
    int rc = check_shape(logN, L, K, dnum);
    if (rc) return rc;
    *bytes = table_total(logN, L, K, dnum);
    return CKKS_OK;
}

static InvScale make_scale(u64 factor, u64 ninv, u64 wlast, u64 m, bool fp) {
    InvScale s;
    s.sx = h_mulmod(ninv, factor, m);
    s.sx_p = h_shoup(s.sx, m);
    s.sy = h_mulmod(h_mulmod(wlast, ninv, m), factor, m);
    s.sy_p = h_shoup(s.sy, m);
    s.sxd = fp ? (double)s.sx : 0.0;
    s.syd = fp ? (double)s.sy : 0.0;
    return s;
}

// (prod of src[k], k != skip) mod m
static u64 prod_except(const std::vector<u64>& src, size_t skip, u64 m) {
    u64 r = 1 % m;
    for (size_t k = 0; k < src.size(); k++)
        if (k != skip) r = h_mulmod(r, src[k] % m, m);
    return r;
}

// Tiles and constant operands of the matrix-core conversion for one digit (conv_mfma_kernel states the layout).
// targets: limb indices of the FpAr targets, in order; mod_of(t): their primes; hat(i, t): (product of the other
// sources) mod that prime, for source i < ns.  Returns the number of tiles written (at most `bound`).
template <class ModFn, class HatFn>
static u32 build_conv_tiles(ConvTile* tiles, u64* aop, u32 bound, u32 ks_n, u32 ns, const std::vector<u32>& targets,
                            ModFn mod_of, HatFn hat) {
    u32 n_tiles = 0;
    for (size_t first = 0; first < targets.size() && n_tiles < bound; n_tiles++) {
        const u32 left = (u32)(targets.size() - first);
        ConvTile& ct = tiles[n_tiles];
        memset(&ct, 0, sizeof(ct));
        ct.ntt = (left > 2 && CKKS_MFMA_NTT == 2) ? 2 : 1;
        const u32 take = left < 2 * ct.ntt ? left : 2 * ct.ntt;
        for (u32 tl = 0; tl < 4; tl++) ct.target[tl] = tl < take ? targets[first + tl] : 0xffffffffu;
        first += take;
        for (u32 ks = 0; ks < ks_n; ks++) {
            for (u32 lane = 0; lane < 64; lane++) {
                const u32 m_row = lane % 32, hk = lane / 32, hrow = (m_row / 4) % 2, a = (m_row / 8) * 4 + m_row % 4;
                const u32 slot = hrow * ct.ntt + a / 8, dg = a % 8;
                for (u32 half = 0; half < 2; half++) {  // the two sources this lane half carries in product ks
                    const u32 i = 4 * ks + 2 * hk + half;
                    u64 word = 0;
                    if (a / 8 < ct.ntt && slot < 4 && ct.target[slot] != 0xffffffffu && i < ns) {
                        const u64 m = mod_of(ct.target[slot]);
                        u64 c = hat(i, ct.target[slot]) % m;  // times 256^bb below
                        for (u32 bb = 0; bb < 8; bb++) {
                            const int64_t centred = c > m / 2 ? (int64_t)c - (int64_t)m : (int64_t)c;
                            const u64 z = (u64)centred + CKKS_DIGIT_BIAS;
                            word |= (u64)((u8_of(z, dg)) ^ 0x80u) << (8 * bb);
                            c = h_mulmod(c, 256 % m, m);
                        }
                    }
                    aop[(((size_t)n_tiles * ks_n + ks) * 64 + lane) * 2 + half] = word;
                }
            }
        }
    }
    return n_tiles;
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
    const size_t total = table_total(logN, L, K, dnum);
    if (table_bytes < total) return CKKS_ENOMEM;
    const SharedLayout lay = shared_layout(logN, L, K);
    const u32 D = L + K, alpha = (L + dnum - 1) / dnum;
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
    const std::vector<u64> specials(c->primes.begin() + L, c->primes.end());

    std::vector<unsigned char> host(total, 0);
    unsigned char* hb = host.data();
    unsigned char* dbase = (unsigned char*)d_tables;
    // ---- block shared by every level
    u64* tw = (u64*)(hb + lay.tw_int);
    double* twf = (double*)(hb + lay.tw_fp);
    PrimeConst* pc = (PrimeConst*)(hb + lay.pc);
    InvScale* sc_plain = (InvScale*)(hb + lay.sc_plain);
    InvScale* sc_dn = (InvScale*)(hb + lay.sc_dn);
    u64* dn_hatinv = (u64*)(hb + lay.dn_hatinv);
    std::vector<u64> pw(N), ninv(D), wlast(D);
    for (u32 i = 0; i < D; i++) {
        const u64 m = c->primes[i];
        const bool fp = m < CKKS_FP_PRIME_LIMIT;
        const u64 psi = h_psi ? h_psi[i] : h_min_root(m, logN);
        c->psi[i] = psi;
        const u64 psi_inv = h_invmod(psi, m);
        u64* fw = tw + (size_t)i * 4 * N;
        double* ff = twf + (size_t)i * 2 * N;
        for (int dir = 0; dir < 2; dir++) {
            const u64 base = dir ? psi_inv : psi;
            pw[0] = 1;
            for (size_t e = 1; e < N; e++) pw[e] = h_mulmod(pw[e - 1], base, m);
            u64* w = fw + (size_t)dir * 2 * N;
            for (size_t k = 0; k < N; k++) {
                w[k] = pw[h_bitrev((u32)k, logN)];
                w[N + k] = h_shoup(w[k], m);
                if (fp) ff[(size_t)dir * N + k] = (double)w[k];
            }
        }
        PrimeConst& p = pc[i];
        p.q = m;
        p.qneg = h_neg_inv64(m);
        p.r1 = (u64)(((u128)1 << 64) % m);
        p.r1_p = h_shoup(p.r1, m);
        p.r2 = h_mulmod(p.r1, p.r1, m);
        p.qd = fp ? (double)m : 0.0;
        p.qinv = fp ? 1.0 / (double)m : 0.0;
        p.fp = fp ? 1 : 0;
        p.pad = 0;
        ninv[i] = h_invmod(N % m, m);
        wlast[i] = fw[2 * N + 1];
        sc_plain[i] = make_scale(1, ninv[i], wlast[i], m, fp);
    }
    for (u32 k = 0; k < K; k++) {  // sources of ModDown: the special limbs, the same at every level
        const u64 pk = specials[k];
        const u64 hinv = h_invmod(prod_except(specials, k, pk), pk);
        dn_hatinv[2 * k] = hinv;
        dn_hatinv[2 * k + 1] = h_shoup(hinv, pk);
        sc_dn[k] = make_scale(hinv, ninv[L + k], wlast[L + k], pk, pc[L + k].fp != 0);
    }
    auto shared_tables = [&](Tables& tb) {
        tb.tw_int = (const u64*)(dbase + lay.tw_int);
        tb.tw_fp = (const double*)(dbase + lay.tw_fp);
        tb.pc = (const PrimeConst*)(dbase + lay.pc);
        tb.sc_plain = (const InvScale*)(dbase + lay.sc_plain);
        tb.sc_dn = (const InvScale*)(dbase + lay.sc_dn);
        tb.dn_hatinv = (const u64*)(dbase + lay.dn_hatinv);
        tb.logN = logN;
    };
    auto classes_mixed = [](const std::vector<u64>& pr) {
        bool any_fp = false, any_int = false;
        for (u64 m : pr) (m < CKKS_FP_PRIME_LIMIT ? any_fp : any_int) = true;
        return any_fp && any_int;
    };

    // ---- one block per level: limb index i of the level is prime ph(i) of the chain
    size_t off = lay.end;
    c->level.resize(L + 1);
    for (u32 ell = 1; ell <= L; ell++) {
        const LevelLayout ll = level_layout(off, ell, K, alpha);
        off = ll.end;
        const u32 Dl = ell + K, beta = (ell + alpha - 1) / alpha;
        auto ph = [&](u32 i) { return i < ell ? i : L + (i - ell); };
        InvScale* sc_up = (InvScale*)(hb + ll.sc_up);
        u64* up_hatinv = (u64*)(hb + ll.up_hatinv);
        u64* up_chat = (u64*)(hb + ll.up_chat);
        double* up_chat_fp = (double*)(hb + ll.up_chat_fp);
        u32* up_fp_ok = (u32*)(hb + ll.up_fp_ok);
        u64* dn_chat = (u64*)(hb + ll.dn_chat);
        double* dn_chat_fp = (double*)(hb + ll.dn_chat_fp);
        u32* dn_fp_ok = (u32*)(hb + ll.dn_fp_ok);
        PinvConst* pinv = (PinvConst*)(hb + ll.pinv);
        u64* pmod = (u64*)(hb + ll.pmod);
        for (u32 j = 0; j < beta; j++) {  // ModUp constants of digit j = limbs [lo, hi)
            const u32 lo = j * alpha, hi = (j + 1) * alpha < ell ? (j + 1) * alpha : ell;
            const std::vector<u64> digit(c->primes.begin() + lo, c->primes.begin() + hi);
            for (u32 i = lo; i < hi; i++) {
                const u64 qi = c->primes[i];
                const u64 hinv = h_invmod(prod_except(digit, i - lo, qi), qi);
                up_hatinv[2 * i] = hinv;
                up_hatinv[2 * i + 1] = h_shoup(hinv, qi);
                sc_up[i] = make_scale(hinv, ninv[i], wlast[i], qi, pc[i].fp != 0);
                for (u32 t = 0; t < Dl; t++) {
                    if (t >= lo && t < hi) continue;
                    const u64 mt = c->primes[ph(t)];
                    const u64 hatb = prod_except(digit, i - lo, mt);
                    up_chat[(size_t)i * Dl + t] = h_mont(hatb, mt);
                    up_chat_fp[(size_t)i * Dl + t] = pc[ph(t)].fp ? (double)hatb : 0.0;
                }
            }
            for (u32 t = 0; t < Dl; t++) {
                bool ok = pc[ph(t)].fp != 0;
                for (u32 i = lo; i < hi; i++) ok = ok && pc[i].fp && c->primes[i] <= 2 * c->primes[ph(t)];
                up_fp_ok[(size_t)j * Dl + t] = ok ? 1 : 0;
            }
        }
        for (u32 i = 0; i < ell; i++) {  // ModDown constants of target q_i
            const u64 qi = c->primes[i];
            for (u32 k = 0; k < K; k++) {
                const u64 hatb = prod_except(specials, k, qi);
                dn_chat[(size_t)k * ell + i] = h_mont(hatb, qi);
                // the conversion kernel strides by ell entries, i.e. 2*ell doubles: index (k*ell + i)*2
                dn_chat_fp[(size_t)k * ell + i] = pc[i].fp ? (double)hatb : 0.0;
            }
            dn_fp_ok[i] = (pc[i].fp && qi >= (1ull << 28)) ? 1 : 0;
            pmod[i] = prod_except(specials, specials.size(), qi);
            const u64 pi = h_invmod(pmod[i], qi);
            pinv[i] = PinvConst{pi, h_shoup(pi, qi), (double)pi};
        }
        // matrix-core conversion: ModUp tiles per digit (FpAr targets outside the digit), ModDown tiles (FpAr q-limbs)
        u32 up_nt = 0, dn_nt = 0;
        const u32 up_ks = mfma_ks_up(alpha), dn_ks = mfma_ks(K), up_bound = mfma_tile_bound(Dl), dn_bound = mfma_tile_bound(ell);
        if (up_ks) {
            for (u32 j = 0; j < beta; j++) {
                const u32 lo = j * alpha, hi = (j + 1) * alpha < ell ? (j + 1) * alpha : ell;
                const std::vector<u64> digit(c->primes.begin() + lo, c->primes.begin() + hi);
                std::vector<u32> tg;
                for (u32 t = 0; t < Dl; t++)
                    if (!(t >= lo && t < hi) && pc[ph(t)].fp) tg.push_back(t);
                const u32 nt = build_conv_tiles((ConvTile*)(hb + ll.up_tiles) + (size_t)j * up_bound,
                                                (u64*)(hb + ll.up_aop) + (size_t)j * up_bound * up_ks * 128, up_bound, up_ks,
                                                hi - lo, tg, [&](u32 t) { return c->primes[ph(t)]; },
                                                [&](u32 i, u32 t) { return prod_except(digit, i, c->primes[ph(t)]); });
                if (nt > up_nt) up_nt = nt;
            }
        }
        if (dn_ks) {
            std::vector<u32> tg;
            for (u32 i = 0; i < ell; i++)
                if (pc[i].fp) tg.push_back(i);
            dn_nt = build_conv_tiles((ConvTile*)(hb + ll.dn_tiles), (u64*)(hb + ll.dn_aop), dn_bound, dn_ks, K, tg,
                                     [&](u32 t) { return c->primes[t]; },
                                     [&](u32 k, u32 t) { return prod_except(specials, k, c->primes[t]); });
        }
        View& v = c->level[ell];
        v.logN = logN, v.L = ell, v.K = K, v.dnum = beta, v.alpha = alpha, v.D = Dl, v.sh = &c->sh;
        v.primes.resize(Dl);
        for (u32 i = 0; i < Dl; i++) v.primes[i] = c->primes[ph(i)];
        v.mixed_classes = classes_mixed(v.primes);
        Tables& tb = v.tb;
        shared_tables(tb);
        tb.sc_up = (const InvScale*)(dbase + ll.sc_up);
        tb.up_hatinv = (const u64*)(dbase + ll.up_hatinv);
        tb.up_chat = (const u64*)(dbase + ll.up_chat);
        tb.up_chat_fp = (const double*)(dbase + ll.up_chat_fp);
        tb.up_fp_ok = (const u32*)(dbase + ll.up_fp_ok);
        tb.dn_chat = (const u64*)(dbase + ll.dn_chat);
        tb.dn_chat_fp = (const double*)(dbase + ll.dn_chat_fp);
        tb.dn_fp_ok = (const u32*)(dbase + ll.dn_fp_ok);
        tb.pinv = (const PinvConst*)(dbase + ll.pinv);
        tb.pmod = (const u64*)(dbase + ll.pmod);
        tb.up_tiles = (const ConvTile*)(dbase + ll.up_tiles), tb.up_aop = (const u64*)(dbase + ll.up_aop);
        tb.dn_tiles = (const ConvTile*)(dbase + ll.dn_tiles), tb.dn_aop = (const u64*)(dbase + ll.dn_aop);
        tb.up_ntiles = up_nt, tb.up_tstride = up_bound, tb.up_ks = up_ks, tb.dn_ntiles = dn_nt, tb.dn_ks = dn_ks;
        tb.L = ell, tb.K = K, tb.dnum = beta, tb.alpha = alpha, tb.D = Dl, tb.Lfull = L, tb.Lq = ell;
    }
    // ---- one block per rescale step: a ModDown whose only "special" prime is q_{ell-1}
    c->rescale.resize(L + 1);
    for (u32 ell = 2; ell <= L; ell++) {
        const RescaleLayout rl = rescale_layout(off, ell);
        off = rl.end;
        const u32 T = ell - 1;
        const u64 ql = c->primes[T];
        InvScale* rsc = (InvScale*)(hb + rl.sc_dn);
        u64* dn_chat = (u64*)(hb + rl.dn_chat);
        double* dn_chat_fp = (double*)(hb + rl.dn_chat_fp);
        u32* dn_fp_ok = (u32*)(hb + rl.dn_fp_ok);
        PinvConst* pinv = (PinvConst*)(hb + rl.pinv);
        rsc[0] = make_scale(1, ninv[T], wlast[T], ql, pc[T].fp != 0);
        for (u32 i = 0; i < T; i++) {
            const u64 qi = c->primes[i];
            dn_chat[i] = h_mont(1, qi);
            dn_chat_fp[i] = pc[i].fp ? 1.0 : 0.0;
            dn_fp_ok[i] = (pc[i].fp && qi >= (1ull << 28)) ? 1 : 0;
            const u64 pi = h_invmod(ql % qi, qi);
            pinv[i] = PinvConst{pi, h_shoup(pi, qi), (double)pi};
        }
        View& v = c->rescale[ell];
        v.logN = logN, v.L = T, v.K = 1, v.dnum = 1, v.alpha = T, v.D = ell, v.sh = &c->sh;
        v.primes.assign(c->primes.begin(), c->primes.begin() + ell);
        v.mixed_classes = classes_mixed(v.primes);
        Tables& tb = v.tb;
        memset(&tb, 0, sizeof(tb));
        shared_tables(tb);
        tb.sc_dn = (const InvScale*)(dbase + rl.sc_dn);
        tb.dn_hatinv = nullptr;
        tb.dn_chat = (const u64*)(dbase + rl.dn_chat);
        tb.dn_chat_fp = (const double*)(dbase + rl.dn_chat_fp);
        tb.dn_fp_ok = (const u32*)(dbase + rl.dn_fp_ok);
        tb.pinv = (const PinvConst*)(dbase + rl.pinv);
        tb.L = T, tb.K = 1, tb.dnum = 1, tb.alpha = T, tb.D = ell, tb.Lfull = ell, tb.Lq = ell;  // phys() is the identity
    }
    // ---- one block per merged ModDown + rescale: sources q_{ell-1}, p_0..p_{K-1} (limbs ell-1 .. of level ell)
    c->merged.resize(L + 1);
    for (u32 ell = 2; K > 0 && ell <= L; ell++) {
        const MergedLayout ml = merged_layout(off, ell, K);
        off = ml.end;
        const u32 T = ell - 1, S = K + 1;
        std::vector<u64> src(1, c->primes[T]);
        src.insert(src.end(), specials.begin(), specials.end());
        auto sph = [&](u32 k) { return k == 0 ? T : L + (k - 1); };  // chain index of source k
        InvScale* msc = (InvScale*)(hb + ml.sc_dn);
        u64* dn_chat = (u64*)(hb + ml.dn_chat);
        double* dn_chat_fp = (double*)(hb + ml.dn_chat_fp);
        u32* dn_fp_ok = (u32*)(hb + ml.dn_fp_ok);
        PinvConst* pinv = (PinvConst*)(hb + ml.pinv);
        for (u32 k = 0; k < S; k++) {
            const u64 sk = src[k];
            const u64 hinv = h_invmod(prod_except(src, k, sk), sk);
            msc[k] = make_scale(hinv, ninv[sph(k)], wlast[sph(k)], sk, pc[sph(k)].fp != 0);
        }
        for (u32 i = 0; i < T; i++) {
            const u64 qi = c->primes[i];
            for (u32 k = 0; k < S; k++) {
                const u64 hatb = prod_except(src, k, qi);
                dn_chat[(size_t)k * T + i] = h_mont(hatb, qi);
                dn_chat_fp[(size_t)k * T + i] = pc[i].fp ? (double)hatb : 0.0;
            }
            dn_fp_ok[i] = (pc[i].fp && qi >= (1ull << 28)) ? 1 : 0;
            const u64 pi = h_invmod(prod_except(src, src.size(), qi), qi);
            pinv[i] = PinvConst{pi, h_shoup(pi, qi), (double)pi};
        }
        u32 dn_nt = 0;
        const u32 dn_ks = mfma_ks(S);
        if (dn_ks) {
            std::vector<u32> tg;
            for (u32 i = 0; i < T; i++)
                if (pc[i].fp) tg.push_back(i);
            dn_nt = build_conv_tiles((ConvTile*)(hb + ml.dn_tiles), (u64*)(hb + ml.dn_aop), mfma_tile_bound(T), dn_ks, S, tg,
                                     [&](u32 t) { return c->primes[t]; },
                                     [&](u32 k, u32 t) { return prod_except(src, k, c->primes[t]); });
        }
        View& v = c->merged[ell];
        v.logN = logN, v.L = T, v.K = S, v.dnum = 1, v.alpha = T, v.D = ell + K, v.sh = &c->sh;
        v.primes = c->level[ell].primes;  // same limb order as the level: q_0..q_{ell-1}, p_0..p_{K-1}
        v.mixed_classes = c->level[ell].mixed_classes;
        Tables& tb = v.tb;
        memset(&tb, 0, sizeof(tb));
        shared_tables(tb);
        tb.sc_dn = (const InvScale*)(dbase + ml.sc_dn);
        tb.dn_hatinv = nullptr;
        tb.dn_chat = (const u64*)(dbase + ml.dn_chat);
        tb.dn_chat_fp = (const double*)(dbase + ml.dn_chat_fp);
        tb.dn_fp_ok = (const u32*)(dbase + ml.dn_fp_ok);
        tb.pinv = (const PinvConst*)(dbase + ml.pinv);
        tb.dn_tiles = (const ConvTile*)(dbase + ml.dn_tiles), tb.dn_aop = (const u64*)(dbase + ml.dn_aop);
        tb.dn_ntiles = dn_nt, tb.dn_ks = dn_ks;
        tb.L = T, tb.K = S, tb.dnum = 1, tb.alpha = T, tb.D = ell + K, tb.Lfull = L, tb.Lq = ell;
    }

    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(d_tables, host.data(), total, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    // this device's copy of the static scratch array (every GPU has its own, at its own address)
    if (e == hipSuccess) e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipGetSymbolAddress(&c->scratch_ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !c->scratch_ptr) {
        (void)hipGetLastError();
        delete c;
        return CKKS_EHIP;
    }
    *out = c;
    return CKKS_OK;
}

extern "C" void ckks_ctx_destroy(ckks_ctx* ctx) {
    if (!ctx) return;
    prof_drain(ctx->sh.prof);
    for (hipEvent_t e : ctx->sh.prof.pool) (void)hipEventDestroy(e);
    if (ctx->sh.side.stream) {
        (void)hipStreamSynchronize(ctx->sh.side.stream);
        (void)hipStreamDestroy(ctx->sh.side.stream);
    }
    for (hipEvent_t e : ctx->sh.side.events) (void)hipEventDestroy(e);
    delete ctx;
}

extern "C" int ckks_profile_enable(ckks_ctx* ctx, int on) {
    if (!ctx) return CKKS_EINVAL;
    prof_drain(ctx->sh.prof);
    ctx->sh.prof.on = on != 0;
    ctx->sh.prof.kinds.clear();
    return CKKS_OK;
}

extern "C" int ckks_profile_read(ckks_ctx* ctx, uint32_t index, const char** name, uint64_t* launches,
                                 double* total_ms, uint64_t* alg_bytes) {
    if (!ctx) return CKKS_EINVAL;
    prof_drain(ctx->sh.prof);
    if (index >= ctx->sh.prof.kinds.size()) return CKKS_EINVAL;
    const ProfKindStat& k = ctx->sh.prof.kinds[index];
    if (name) *name = k.name.c_str();
    if (launches) *launches = k.launches;
    if (total_ms) *total_ms = k.ms;
    if (alg_bytes) *alg_bytes = k.bytes;
    return CKKS_OK;
}

extern "C" int ckks_set_overlap(ckks_ctx* ctx, int on) {
    if (!ctx) return CKKS_EINVAL;
    if (ctx->sh.side.active) return fail(ctx, CKKS_EINVAL, "cannot change overlap inside an operation");
    ctx->sh.side.enabled = on != 0;
    return CKKS_OK;
}

extern "C" const char* ckks_last_error(const ckks_ctx* ctx) { return ctx ? ctx->sh.err.c_str() : "null context"; }

extern "C" uint64_t ckks_ctx_psi(const ckks_ctx* ctx, uint32_t i) { return (ctx && i < ctx->D) ? ctx->psi[i] : 0; }

// ----------------------------------------------------------------------------- launches
static inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

static int hip_check(const View* c, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        c->sh->err = std::string(what) + ": " + hipGetErrorString(e);
        return CKKS_EHIP;
    }
    return CKKS_OK;
}

// grid of an XCD-aware launch: groups padded to a multiple of 8, times the instances per group
static inline u32 xcd_grid(u32 groups, u32 inst) { return ((groups + 7) / 8) * 8 * inst; }
static inline u32 tiles_of(const View* c) { return (1u << (c->logN - 8)) / 16; }

// Maximal runs of consecutive primes [lo, hi) that share an arithmetic (FpAr / IntAr).
struct ClassRun {
    u32 first, count;
    bool fp;
};
static std::vector<ClassRun> class_runs(const View* c, u32 lo, u32 hi) {
    std::vector<ClassRun> r;
    for (u32 i = lo; i < hi; i++) {
        const bool fp = c->primes[i] < CKKS_FP_PRIME_LIMIT;
        if (!r.empty() && r.back().fp == fp) r.back().count++;
        else r.push_back(ClassRun{i, 1, fp});
    }
    return r;
}

// A launcher type L provides
//   template <class AR, int A> static void go(grid, stream, args, tables, run)   the launch
//   static std::string name(const char* ar, int A)                               the profiler's kernel name
template <class L, class ArgT>
static void dispatch_kernel(const View* c, bool fp, dim3 grid, hipStream_t s, const ArgT& a, LimbRun run) {
#define CKKS_CASE_A(AV)                                               \
    case AV:                                                          \
        if (fp) L::template go<FpAr, AV>(grid, s, a, c->tb, run);     \
        else L::template go<IntAr, AV>(grid, s, a, c->tb, run);       \
        break;
    switch (c->logN - 8) {
        CKKS_CASE_A(4)
        CKKS_CASE_A(5)
        CKKS_CASE_A(6)
        CKKS_CASE_A(7)
        CKKS_CASE_A(8)
    }
#undef CKKS_CASE_A
}

static std::string kname(const char* base, const char* ar, int A, const char* tail) {
    return std::string(base) + "<" + ar + ", " + std::to_string(A) + tail + ">";
}

// One launch per arithmetic run of the primes [lo, hi).  limb_base converts a prime index into the
// kernel's limb index.  by_limb: groups = run limbs x groups_n, instances = inst_n; otherwise
// (conversion targets): groups = groups_n, instances = the run's limbs in blocks of inst_n.  alg(first, count) gives
// the algorithmic limbs (read + written once) of the launch covering primes [first, first+count).
// only: -1 = every run, 0 = IntAr runs only, 1 = FpAr runs only.
template <class L, class ArgT, class AlgFn>
static void launch_runs(const View* c, u32 lo, u32 hi, u32 limb_base, bool by_limb, u32 groups_n, u32 inst_n,
                        const ArgT& a, hipStream_t s, AlgFn alg, int only = -1) {
    for (const ClassRun& cr : class_runs(c, lo, hi)) {
        if (only >= 0 && (int)cr.fp != only) continue;
        const LimbRun run = {cr.first - limb_base, cr.count};
        // conversion launches: inst_n holds the targets per workgroup of FpAr runs in its low half and of
        // IntAr runs in its high half
        const u32 tbn = cr.fp ? (inst_n & 0xffff) : (inst_n >> 16);
        const dim3 grid(by_limb ? xcd_grid(cr.count * groups_n, inst_n)
                                : xcd_grid(groups_n, (cr.count + tbn - 1) / tbn));
        hipStream_t rs = (!cr.fp && c->sh->side.active) ? c->sh->side.stream : s;
        ProfScope ps(c, c->sh->prof.on ? L::name(cr.fp ? "FpAr" : "IntAr", (int)c->logN - 8) : std::string(),
                     c->sh->prof.on ? alg(cr.first, cr.count) : 0, rs);
        dispatch_kernel<L>(c, cr.fp, grid, rs, a, run);
    }
}

template <int LOAD>
struct InvContigL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const InvContigArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((inv_contig_kernel<AR, A, LOAD>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) {
        return kname("inv_contig_kernel", ar, A, LOAD == 0 ? ", 0" : LOAD == 1 ? ", 1" : ", 2");
    }
};
struct InvStridedL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const InvStridedArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((inv_strided_kernel<AR, A>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) { return kname("inv_strided_kernel", ar, A, ""); }
};
struct FwdStridedL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const FwdStridedArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((fwd_strided_kernel<AR, A>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) { return kname("fwd_strided_kernel", ar, A, ""); }
};
// target limbs converted per workgroup, per direction and arithmetic (measured optimum: more targets save L2
// reads and conversions of the sources but cost registers; 4 FP64 or 3 integer targets are slower again)
#ifndef CKKS_CONV_TB_UP_FP
#define CKKS_CONV_TB_UP_FP 3
#endif
#ifndef CKKS_CONV_TB_DN_FP
#define CKKS_CONV_TB_DN_FP 3
#endif
#ifndef CKKS_CONV_TB_INT
#define CKKS_CONV_TB_INT 2
#endif
template <int DIR, bool FP>
struct ConvTB {
    static constexpr int value = FP ? (DIR == CONV_UP ? CKKS_CONV_TB_UP_FP : CKKS_CONV_TB_DN_FP) : CKKS_CONV_TB_INT;
};
// DG: the sources are digit-format words (only where the FpAr targets of the view go to the matrix-core kernel, so
// only integer-arithmetic runs are launched with it)
template <int DIR, bool DG>
struct ConvL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const ConvArgs& a, const Tables& tb, LimbRun run) {
        if constexpr (!(AR::is_fp && DG))
            hipLaunchKernelGGL((conv_fwd_strided_kernel<AR, A, DIR, ConvTB<DIR, AR::is_fp>::value, DG>), g, dim3(256), 0, s, a, tb,
                               run);
    }
    static std::string name(const char* ar, int A) {
        const int tbv = ar[0] == 'F' ? ConvTB<DIR, true>::value : ConvTB<DIR, false>::value;
        return kname("conv_fwd_strided_kernel", ar, A,
                     (std::string(", ") + std::to_string(DIR) + ", " + std::to_string(tbv) + (DG ? ", true" : ", false")).c_str());
    }
};
struct FwdContigL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const FwdContigArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((fwd_contig_kernel<AR, A>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) { return kname("fwd_contig_kernel", ar, A, ""); }
};
template <int OWN, bool HOISTED, bool FUSED>
struct KsInnerL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const InnerArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((ks_inner_kernel<AR, A, OWN, HOISTED, FUSED>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) {
        return kname("ks_inner_kernel", ar, A,
                     (std::string(", ") + std::to_string(OWN) + (HOISTED ? ", true" : ", false") + (FUSED ? ", true" : ", false"))
                         .c_str());
    }
};
template <int MODE>
struct KsFinalL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const FinalArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((ks_final_kernel<AR, A, MODE>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int A) {
        return kname("ks_final_kernel", ar, A, (std::string(", ") + std::to_string(MODE)).c_str());
    }
};

template <int LOAD>
static void launch_inv_contig(const View* c, const InvContigArgs& a, hipStream_t s) {
    const u32 pb = a.sel.prime_base;
    const u64 per = (u64)a.sel.n_inst * (LOAD == INV_TENSOR ? 3 : 2);
    launch_runs<InvContigL<LOAD>>(c, pb, pb + a.sel.n_l, pb, true, tiles_of(c), a.sel.n_inst, a, s,
                                  [per](u32, u32 n) { return per * n; });
}

static void launch_inv_strided(const View* c, const InvStridedArgs& a, hipStream_t s) {
    const u32 pb = a.sel.prime_base;
    const u64 per = (u64)a.sel.n_inst * 2;
    launch_runs<InvStridedL>(c, pb, pb + a.sel.n_l, pb, true, tiles_of(c), a.sel.n_inst, a, s,
                             [per](u32, u32 n) { return per * n; });
}

static void launch_fwd_strided(const View* c, const FwdStridedArgs& a, hipStream_t s) {
    const u32 pb = a.sel.prime_base;
    const u64 per = (u64)a.sel.n_inst * 2;
    launch_runs<FwdStridedL>(c, pb, pb + a.sel.n_l, pb, true, tiles_of(c), a.sel.n_inst, a, s,
                             [per](u32, u32 n) { return per * n; });
}

template <int A, int DIR>
static void launch_conv_mfma_ks(const View* c, u32 ks, dim3 grid, hipStream_t s, const MfmaConvArgs& a) {
    switch (ks) {
        case 1: hipLaunchKernelGGL((conv_mfma_kernel<A, 1, DIR, CKKS_MFMA_NTT>), grid, dim3(256), 0, s, a, c->tb); break;
        case 2: hipLaunchKernelGGL((conv_mfma_kernel<A, 2, DIR, CKKS_MFMA_NTT>), grid, dim3(256), 0, s, a, c->tb); break;
    }
}

// conversion of every FpAr target on the matrix cores (the view's tile tables say which targets those are)
template <int DIR>
static void launch_conv_mfma(const View* c, const ConvArgs& a, hipStream_t s) {
    const Tables& tb = c->tb;
    MfmaConvArgs m;
    m.src = a.src, m.dst = a.dst, m.groups_outer = a.groups_outer;
    m.tiles = DIR == CONV_UP ? tb.up_tiles : tb.dn_tiles;
    m.aop = DIR == CONV_UP ? tb.up_aop : tb.dn_aop;
    m.n_tiles = DIR == CONV_UP ? tb.up_ntiles : tb.dn_ntiles;
    m.tile_stride = DIR == CONV_UP ? tb.up_tstride : tb.dn_ntiles;
    const u32 ks = DIR == CONV_UP ? tb.up_ks : tb.dn_ks;
    const u32 groups = a.groups_outer * (DIR == CONV_UP ? c->dnum : 1) * tiles_of(c);
    const dim3 grid(xcd_grid(groups, m.n_tiles));
    u64 limbs = 0;  // FpAr targets written (per digit that does not own them) plus the sources, read once
    if (c->sh->prof.on) {
        const u32 hi = DIR == CONV_UP ? c->D : c->L;
        for (u32 t = 0; t < hi; t++)
            if (c->primes[t] < CKKS_FP_PRIME_LIMIT) limbs += DIR == CONV_UP ? c->dnum - (t < c->L ? 1 : 0) : 1;
        limbs = (u64)a.groups_outer * (limbs + (DIR == CONV_UP ? c->L : c->K));
    }
    ProfScope ps(c, c->sh->prof.on ? std::string("conv_mfma_kernel<") + std::to_string((int)c->logN - 8) + ", " + std::to_string(ks) +
                                         ", " + std::to_string(DIR) + ", " + std::to_string(CKKS_MFMA_NTT) + ">"
                                   : std::string(),
                 limbs, s);
    switch (c->logN - 8) {
        case 4: launch_conv_mfma_ks<4, DIR>(c, ks, grid, s, m); break;
        case 5: launch_conv_mfma_ks<5, DIR>(c, ks, grid, s, m); break;
        case 6: launch_conv_mfma_ks<6, DIR>(c, ks, grid, s, m); break;
        case 7: launch_conv_mfma_ks<7, DIR>(c, ks, grid, s, m); break;
        case 8: launch_conv_mfma_ks<8, DIR>(c, ks, grid, s, m); break;
    }
}

static inline bool conv_on_matrix_cores(const View* c, int dir) {
    return dir == CONV_UP ? c->tb.up_ntiles != 0 : c->tb.dn_ntiles != 0;
}

// cls: -1 = every target, 0 = IntAr targets only, 1 = FpAr targets only
template <int DIR>
static void launch_conv(const View* c, const ConvArgs& a, hipStream_t s, int cls = -1) {
    const u64 outer = a.groups_outer;
    const bool mfma = conv_on_matrix_cores(c, DIR);  // FpAr targets go to the matrix-core kernel when the view has tiles
    if (mfma && cls != 0) launch_conv_mfma<DIR>(c, a, s);
    if (mfma && cls == 1) return;
    const int only = mfma ? 0 : cls;
    const u32 tbs = ConvTB<DIR, true>::value | (ConvTB<DIR, false>::value << 16);
    if (DIR == CONV_UP) {  // groups = (batch, digit, tile); instances = blocks of the run's target primes
        auto alg = [c, outer](u32 first, u32 n) {
            u64 w = 0;  // every target limb is written for each digit that does not own it
            for (u32 t = first; t < first + n; t++) w += c->dnum - (t < c->L ? 1 : 0);
            return outer * (w + c->L);  // plus the source coefficients, read once
        };
        const u32 groups = a.groups_outer * c->dnum * tiles_of(c);
        if (a.src_fmt == SRC_DIGITS) launch_runs<ConvL<DIR, true>>(c, 0, c->D, 0, false, groups, tbs, a, s, alg, only);
        else launch_runs<ConvL<DIR, false>>(c, 0, c->D, 0, false, groups, tbs, a, s, alg, only);
    } else {  // groups = (g, tile); instances = blocks of the run's target q-limbs
        auto alg = [c, outer](u32, u32 n) { return outer * (n + (u64)c->K); };
        const u32 groups = a.groups_outer * tiles_of(c);
        if (a.src_fmt == SRC_DIGITS) launch_runs<ConvL<DIR, true>>(c, 0, c->L, 0, false, groups, tbs, a, s, alg, only);
        else launch_runs<ConvL<DIR, false>>(c, 0, c->L, 0, false, groups, tbs, a, s, alg, only);
    }
}

static void launch_fwd_contig(const View* c, const FwdContigArgs& a, hipStream_t s) {
    const u32 pb = a.sel.prime_base;
    const u64 per = (u64)a.sel.n_inst * 2;
    launch_runs<FwdContigL>(c, pb, pb + a.sel.n_l, pb, true, tiles_of(c), a.sel.n_inst, a, s,
                            [per](u32, u32 n) { return per * n; });
}

// limbs [lo, hi) of the extended basis.  FUSED: the launch also ends the ModDown on its limbs (all below
// a.split, after the conversion of the special part) and writes the result instead of c'.
template <int OWN, bool HOISTED, bool FUSED = false>
static void launch_ks_inner(const View* c, const InnerArgs& a, hipStream_t s, u32 lo, u32 hi) {
    const u64 n_inst = a.n_inst;
    launch_runs<KsInnerL<OWN, HOISTED, FUSED>>(
        c, lo, hi, 0, true, tiles_of(c), a.n_inst, a, s, [c, n_inst](u32 first, u32 n) {
            u64 limbs = 0;
            for (u32 i = first; i < first + n; i++) {
                const bool q = i < c->L;
                limbs += n_inst * ((u64)c->dnum - (q ? 1 : 0)            // extended digits outside their own limbs
                                   + (q ? (OWN == OWN_TENSOR ? 4 : 1) : 0)  // the switched polynomial (HMult: both inputs) on its own limb
                                   + 2                                     // c' (or the result) written
                                   + (FUSED ? 2 + (OWN == OWN_ROT ? 1 : 0) : 0))  // converted special part (+ sigma_g(b))
                         + (HOISTED ? n_inst : 1) * 2 * (u64)c->dnum;      // key limbs
            }
            return limbs;
        });
}
template <int OWN, bool HOISTED>
static void launch_ks_inner(const View* c, const InnerArgs& a, hipStream_t s) {
    launch_ks_inner<OWN, HOISTED, false>(c, a, s, 0, c->D);
}

#define CKKS_DH_EPT 4
struct DhAccumL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const DhInnerArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((dh_accum_kernel<AR, CKKS_DH_EPT>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int) {
        return std::string("dh_accum_kernel<") + ar + ", " + std::to_string(CKKS_DH_EPT) + ">";
    }
};

struct BsgsMacL {
    template <class AR, int A>
    static void go(dim3 g, hipStream_t s, const BsgsMacArgs& a, const Tables& tb, LimbRun run) {
        hipLaunchKernelGGL((bsgs_mac_kernel<AR, CKKS_DH_EPT>), g, dim3(256), 0, s, a, tb, run);
    }
    static std::string name(const char* ar, int) {
        return std::string("bsgs_mac_kernel<") + ar + ", " + std::to_string(CKKS_DH_EPT) + ">";
    }
};

static void launch_bsgs_mac(const View* c, const BsgsMacArgs& a, hipStream_t s) {
    const u32 chunks = (1u << c->logN) / (256 * CKKS_DH_EPT);
    for (const ClassRun& cr : class_runs(c, 0, c->D)) {
        const LimbRun run = {cr.first, cr.count};
        hipStream_t rs = (!cr.fp && c->sh->side.active) ? c->sh->side.stream : s;
        // per limb and giant step: n1 rotations (2 components) and n1 plaintexts read, 2 components written
        ProfScope ps(c, c->sh->prof.on ? BsgsMacL::name(cr.fp ? "FpAr" : "IntAr", 0) : std::string(),
                     (u64)cr.count * a.n2 * (3 * (u64)a.n1 + 2), rs);
        dispatch_kernel<BsgsMacL>(c, cr.fp, dim3(xcd_grid(cr.count * chunks, a.n2)), rs, a, run);
    }
}

// one workgroup per 256 * CKKS_DH_EPT slots of a limb, all limbs of the extended basis
static void launch_dh_accum(const View* c, const DhInnerArgs& a, hipStream_t s) {
    const u64 n_rot = a.n_rot, acc = a.accumulate ? 2 : 0, dnum = c->dnum;
    const u32 chunks = (1u << c->logN) / (256 * CKKS_DH_EPT);
    for (const ClassRun& cr : class_runs(c, 0, c->D)) {
        const LimbRun run = {cr.first, cr.count};
        u64 limbs = 0;  // per limb and rotation: the digits, the plaintext, both key components (and b on q-limbs); C_t written
        for (u32 i = cr.first; i < cr.first + cr.count; i++) limbs += n_rot * (3 * dnum + 1 + (i < c->L ? 1 : 0)) + 2 + acc;
        hipStream_t rs = (!cr.fp && c->sh->side.active) ? c->sh->side.stream : s;
        ProfScope ps(c, c->sh->prof.on ? DhAccumL::name(cr.fp ? "FpAr" : "IntAr", 0) : std::string(), limbs, rs);
        dispatch_kernel<DhAccumL>(c, cr.fp, dim3(cr.count * chunks), rs, a, run);
    }
}

template <int MODE>
static void launch_ks_final(const View* c, const FinalArgs& a, hipStream_t s) {
    u64 per;  // algorithmic limbs per q-limb
    if (MODE == FIN_HOISTED) per = (u64)a.n_rot * (2 + 2 + 1 + 1) + (2 + (a.accumulate ? 2 : 0));
    else per = (u64)a.n_inst * 6;
    launch_runs<KsFinalL<MODE>>(c, 0, c->L, 0, true, tiles_of(c), a.n_inst, a, s, [per](u32, u32 n) { return per * n; });
}

template <int AL>
static void launch_modup_a(const View* c, const u64* in, u64* out, u32 batch, hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, c->dnum, batch), block(256);
    ProfScope ps(c, std::string("modup_kernel"), (u64)batch * (2 * (u64)c->L + (u64)c->dnum * (c->D - c->alpha)), s);
    hipLaunchKernelGGL(modup_kernel<AL>, grid, block, 0, s, in, out, c->tb);
}
static void launch_modup(const View* c, const u64* in, u64* out, u32 batch, hipStream_t s) {
    switch (c->alpha) {
        case 1: launch_modup_a<1>(c, in, out, batch, s); break;
        case 2: launch_modup_a<2>(c, in, out, batch, s); break;
        case 3: launch_modup_a<3>(c, in, out, batch, s); break;
        case 4: launch_modup_a<4>(c, in, out, batch, s); break;
        case 5: launch_modup_a<5>(c, in, out, batch, s); break;
        case 6: launch_modup_a<6>(c, in, out, batch, s); break;
        case 7: launch_modup_a<7>(c, in, out, batch, s); break;
        case 8: launch_modup_a<8>(c, in, out, batch, s); break;
        case 9: launch_modup_a<9>(c, in, out, batch, s); break;
        case 10: launch_modup_a<10>(c, in, out, batch, s); break;
        case 11: launch_modup_a<11>(c, in, out, batch, s); break;
        case 12: launch_modup_a<12>(c, in, out, batch, s); break;
        case 13: launch_modup_a<13>(c, in, out, batch, s); break;
        case 14: launch_modup_a<14>(c, in, out, batch, s); break;
        case 15: launch_modup_a<15>(c, in, out, batch, s); break;
        case 16: launch_modup_a<16>(c, in, out, batch, s); break;
    }
}

template <int KK>
static void launch_moddown_k(const View* c, const u64* in, u64* out, u32 groups, hipStream_t s) {
    const dim3 grid((1u << c->logN) / 256, groups), block(256);
    ProfScope ps(c, std::string("moddown_kernel"), (u64)groups * (c->K + 2 * (u64)c->L), s);
    hipLaunchKernelGGL(moddown_kernel<KK>, grid, block, 0, s, in, out, c->tb);
}
static void launch_moddown(const View* c, const u64* in, u64* out, u32 groups, hipStream_t s) {
    switch (c->K) {
        case 1: launch_moddown_k<1>(c, in, out, groups, s); break;
        case 2: launch_moddown_k<2>(c, in, out, groups, s); break;
        case 3: launch_moddown_k<3>(c, in, out, groups, s); break;
        case 4: launch_moddown_k<4>(c, in, out, groups, s); break;
        case 5: launch_moddown_k<5>(c, in, out, groups, s); break;
        case 6: launch_moddown_k<6>(c, in, out, groups, s); break;
        case 7: launch_moddown_k<7>(c, in, out, groups, s); break;
        case 8: launch_moddown_k<8>(c, in, out, groups, s); break;
        case 9: launch_moddown_k<9>(c, in, out, groups, s); break;
        case 10: launch_moddown_k<10>(c, in, out, groups, s); break;
        case 11: launch_moddown_k<11>(c, in, out, groups, s); break;
        case 12: launch_moddown_k<12>(c, in, out, groups, s); break;
        case 13: launch_moddown_k<13>(c, in, out, groups, s); break;
        case 14: launch_moddown_k<14>(c, in, out, groups, s); break;
        case 15: launch_moddown_k<15>(c, in, out, groups, s); break;
        case 16: launch_moddown_k<16>(c, in, out, groups, s); break;
    }
}

// ---------------------------------------------------------------------- workspace carving
// x  [xg][L][N]        coefficients of the switched polynomial (raw after pass 1, then canonical * pre-factor)
// dt [dg][dnum][D][N]  extended digits (first forward pass done; own-digit limbs unused)
// cq [cg][2][L][N]     c' on the q-limbs, canonical evaluation form
// cp [cg][2][K][N]     c' on the special limbs: raw after the first inverse pass, then coefficients * pre-factor
// cv [cg][2][L][N]     Conv_{P->Q} of the special part, first forward pass done
struct Workspace {
    u64 *x, *dt, *cq, *cp, *cv;
};

// with_cq = false: the plain key-switch pipeline, whose c' on the q-limbs never leaves the registers of the kernel
// that accumulates it: no cq (a fifth of the workspace at (24,6,4))
static size_t ks_workspace_words(const View* c, u32 xg, u32 dg, u32 cg, bool with_cq = true) {
    const size_t N = (size_t)1 << c->logN;
    return ((size_t)xg * c->L + (size_t)dg * c->dnum * c->D + (size_t)cg * 2 * ((with_cq ? 2 : 1) * (size_t)c->L + c->K)) * N;
}

static Workspace carve(const View* c, void* ws, u32 xg, u32 dg, u32 cg, bool with_cq = true) {
    const size_t N = (size_t)1 << c->logN;
    Workspace w;
    w.x = (u64*)ws;
    w.dt = w.x + (size_t)xg * c->L * N;
    w.cq = w.dt + (size_t)dg * c->dnum * c->D * N;
    w.cp = w.cq + (with_cq ? (size_t)cg * 2 * c->L * N : 0);
    w.cv = w.cp + (size_t)cg * 2 * c->K * N;
    if (!with_cq) w.cq = nullptr;
    return w;
}

static int view_workspace_bytes(const View* v, int op, uint32_t batch_or_nrot, size_t* bytes) {
    if (batch_or_nrot == 0) return fail(v, CKKS_EINVAL, "batch must be positive");
    switch (op) {
        case CKKS_OP_NTT:
        case CKKS_OP_MODUP:
        case CKKS_OP_MODDOWN:
        case CKKS_OP_AUTOMORPH: *bytes = 0; return CKKS_OK;
        case CKKS_OP_KEYSWITCH:
        case CKKS_OP_HMULT_RELIN:
        case CKKS_OP_HROT:
            if (v->K == 0) return fail(v, CKKS_EUNSUPPORTED, "context has no special primes");
            *bytes = ks_workspace_words(v, batch_or_nrot, batch_or_nrot, batch_or_nrot, false) * sizeof(u64);
            return CKKS_OK;
        case CKKS_OP_HROT_HOISTED_MAC: {
            if (v->K == 0) return fail(v, CKKS_EUNSUPPORTED, "context has no special primes");
            const u32 chunk = batch_or_nrot < CKKS_ROT_CHUNK ? batch_or_nrot : CKKS_ROT_CHUNK;
            *bytes = ks_workspace_words(v, 1, 1, chunk) * sizeof(u64);
            return CKKS_OK;
        }
        case CKKS_OP_HROT_DH_MAC:
            if (v->K == 0) return fail(v, CKKS_EUNSUPPORTED, "context has no special primes");
            *bytes = ks_workspace_words(v, 1, 1, 1) * sizeof(u64);
            return CKKS_OK;
        case CKKS_OP_RESCALE:  // last-limb coefficients [b][2][N] + converted part [b][2][ell-1][N]
            if (v->L < 2) return fail(v, CKKS_EINVAL, "rescale needs at least two limbs");
            *bytes = ((size_t)batch_or_nrot * 2 * v->L * sizeof(u64)) << v->logN;
            return CKKS_OK;
    }
    return fail(v, CKKS_EINVAL, "unknown op selector");
}

static const View* view_at(const ckks_ctx* ctx, uint32_t level) {
    if (level == 0 || level > ctx->L) {
        ctx->sh.err = "level must be between 1 and L";
        return nullptr;
    }
    return &ctx->level[level];
}

extern "C" int ckks_workspace_bytes_at(const ckks_ctx* ctx, int op, uint32_t level, uint32_t batch_or_nrot,
                                       size_t* bytes) {
    if (!ctx || !bytes) return CKKS_EINVAL;
    const View* v = view_at(ctx, level);
    if (!v) return CKKS_EINVAL;
    return view_workspace_bytes(v, op, batch_or_nrot, bytes);
}

extern "C" int ckks_workspace_bytes(const ckks_ctx* ctx, int op, uint32_t batch_or_nrot, size_t* bytes) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_workspace_bytes_at(ctx, op, ctx->L, batch_or_nrot, bytes);
}

// --------------------------------------------------------------------------- entry points
static int check_limb_range(const View* c, u32 prime_first, u32 n_limbs, u32 batch) {
    if (n_limbs == 0 || batch == 0) return fail(c, CKKS_EINVAL, "n_limbs and batch must be positive");
    if ((u64)prime_first + n_limbs > c->D) return fail(c, CKKS_EINVAL, "limb range exceeds the prime chain");
    if ((u64)n_limbs * batch > (1u << 20)) return fail(c, CKKS_EINVAL, "batch too large");
    return CKKS_OK;
}

static int ntt_entry(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                     void* stream, bool inverse) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = ctx->full();
    if (!d_x || misaligned(d_x, 16)) return fail(c, CKKS_EINVAL, "d_x is null or not 16-byte aligned");
    int rc = check_limb_range(c, prime_first, n_limbs, batch);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const LimbSel sel = {n_limbs, batch, n_limbs, 0, prime_first, 0};
    if (!inverse) {
        FwdStridedArgs a1 = {d_x, d_x, sel};
        launch_fwd_strided(c, a1, s);
        FwdContigArgs a2 = {d_x, sel};
        launch_fwd_contig(c, a2, s);
    } else {
        InvContigArgs a1 = {d_x, nullptr, d_x, sel, sel, {1}, 0};
        launch_inv_contig<INV_PLAIN>(c, a1, s);
        InvStridedArgs a2 = {d_x, sel, SC_PLAIN, 0};
        launch_inv_strided(c, a2, s);
    }
    return hip_check(c, inverse ? "ckks_intt" : "ckks_ntt");
}

extern "C" int ckks_ntt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                        void* stream) {
    return ntt_entry(ctx, d_x, prime_first, n_limbs, batch, stream, false);
}

extern "C" int ckks_intt(ckks_ctx* ctx, uint64_t* d_x, uint32_t prime_first, uint32_t n_limbs, uint32_t batch,
                         void* stream) {
    return ntt_entry(ctx, d_x, prime_first, n_limbs, batch, stream, true);
}

static int check_ks_ctx(const View* c, u32 batch) {
    if (c->K == 0) return fail(c, CKKS_EUNSUPPORTED, "context has no special primes");
    if (batch == 0 || batch > 4096) return fail(c, CKKS_EINVAL, "batch out of range");
    return CKKS_OK;
}

extern "C" int ckks_modup(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = ctx->full();
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(c, batch);
    if (rc) return rc;
    launch_modup(c, d_in, d_out, batch, (hipStream_t)stream);
    return hip_check(c, "ckks_modup");
}

extern "C" int ckks_moddown(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = ctx->full();
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(c, batch);
    if (rc) return rc;
    launch_moddown(c, d_in, d_out, batch, (hipStream_t)stream);
    return hip_check(c, "ckks_moddown");
}

static int check_galois(const View* c, u32 g) {
    if ((g & 1) == 0 || g >= (2u << c->logN)) return fail(c, CKKS_EINVAL, "Galois element must be odd and below 2N");
    return CKKS_OK;
}

extern "C" int ckks_automorph(ckks_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, uint32_t prime_first,
                              uint32_t n_limbs, uint32_t galois, int eval_domain, uint32_t batch, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = ctx->full();
    if (!d_in || !d_out || misaligned(d_in, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (d_in == d_out) return fail(c, CKKS_EINVAL, "automorphism cannot run in place");
    int rc = check_limb_range(c, prime_first, n_limbs, batch);
    if (rc) return rc;
    rc = check_galois(c, galois);
    if (rc) return rc;
    if (batch > 65535) return fail(c, CKKS_EINVAL, "batch too large");
    const dim3 grid((1u << c->logN) / 256, n_limbs, batch), block(256);
    hipStream_t s = (hipStream_t)stream;
    ProfScope ps(c, std::string(eval_domain ? "automorph_eval_kernel" : "automorph_coeff_kernel"), (u64)batch * n_limbs * 2, s);
    if (eval_domain) {
        hipLaunchKernelGGL(automorph_eval_kernel, grid, block, 0, s, d_in, d_out, c->logN, n_limbs, galois);
    } else {
        // inverse of g modulo 2N (a power of two): Newton iteration on 32-bit words, then mask
        u32 inv = galois;
        for (int i = 0; i < 5; i++) inv *= 2 - galois * inv;
        inv &= (2u << c->logN) - 1;
        hipLaunchKernelGGL(automorph_coeff_kernel, grid, block, 0, s, d_in, d_out, c->tb.pc, c->logN, n_limbs,
                           prime_first, inv);
    }
    return hip_check(c, "ckks_automorph");
}

extern "C" int ckks_pointwise(ckks_ctx* ctx, int op, const uint64_t* d_a, const uint64_t* d_b, uint64_t* d_out,
                              uint32_t prime_first, uint32_t n_limbs, uint32_t batch, uint32_t b_period, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = ctx->full();
    if (!d_a || !d_b || !d_out || misaligned(d_a, 16) || misaligned(d_b, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (op < CKKS_PW_ADD || op > CKKS_PW_MAC) return fail(c, CKKS_EINVAL, "unknown limb-wise operation");
    int rc = check_limb_range(c, prime_first, n_limbs, batch);
    if (rc) return rc;
    if (batch > 65535) return fail(c, CKKS_EINVAL, "batch too large");
    if (b_period == 0 || b_period > batch) return fail(c, CKKS_EINVAL, "b_period must be in 1..batch");
    const dim3 grid((1u << c->logN) / 512, n_limbs, batch), block(256);
    hipStream_t s = (hipStream_t)stream;
    static const char* const names[4] = {"pointwise_kernel<add>", "pointwise_kernel<sub>", "pointwise_kernel<mul>",
                                         "pointwise_kernel<mac>"};
    ProfScope ps(c, std::string(names[op]), (u64)batch * n_limbs * (op == CKKS_PW_MAC ? 3 : 2) + (u64)b_period * n_limbs, s);
    switch (op) {
        case CKKS_PW_ADD:
            hipLaunchKernelGGL(pointwise_kernel<PW_ADD>, grid, block, 0, s, d_a, d_b, d_out, c->tb.pc, c->logN, n_limbs,
                               prime_first, b_period);
            break;
        case CKKS_PW_SUB:
            hipLaunchKernelGGL(pointwise_kernel<PW_SUB>, grid, block, 0, s, d_a, d_b, d_out, c->tb.pc, c->logN, n_limbs,
                               prime_first, b_period);
            break;
        case CKKS_PW_MUL:
            hipLaunchKernelGGL(pointwise_kernel<PW_MUL>, grid, block, 0, s, d_a, d_b, d_out, c->tb.pc, c->logN, n_limbs,
                               prime_first, b_period);
            break;
        default:
            hipLaunchKernelGGL(pointwise_kernel<PW_MAC>, grid, block, 0, s, d_a, d_b, d_out, c->tb.pc, c->logN, n_limbs,
                               prime_first, b_period);
            break;
    }
    return hip_check(c, "ckks_pointwise");
}

// [p, p + bytes) ranges that share at least one byte
static inline bool ranges_overlap(const void* a, size_t a_bytes, const void* b, size_t b_bytes) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a && b && a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}
// The kernels of a call read the inputs (permuted gathers, tensor terms, later chunks of rotations) after the
// first words of the output have been written, so an output that shares memory with an input, or an output or
// input that shares memory with the workspace, gives wrong words without any error: rejected here.
static int check_no_alias(const View* c, const void* out, size_t out_bytes, const void* in1, size_t in1_bytes,
                          const void* in2, size_t in2_bytes, const void* ws, size_t ws_bytes) {
    if (ranges_overlap(out, out_bytes, in1, in1_bytes) || ranges_overlap(out, out_bytes, in2, in2_bytes))
        return fail(c, CKKS_EINVAL, "output overlaps an input");
    if (ranges_overlap(out, out_bytes, ws, ws_bytes) || ranges_overlap(in1, in1_bytes, ws, ws_bytes) ||
        ranges_overlap(in2, in2_bytes, ws, ws_bytes))
        return fail(c, CKKS_EINVAL, "workspace overlaps an operand");
    return CKKS_OK;
}
static inline size_t limb_bytes(const View* c, size_t limbs) { return (limbs * sizeof(u64)) << c->logN; }

static int check_ks_args(const View* c, const void* a, const void* b, const void* out, u32 batch, int op,
                         const void* ws, size_t ws_bytes) {
    if (!a || !b || !out || misaligned(a, 16) || misaligned(b, 16) || misaligned(out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_ctx(c, batch);
    if (rc) return rc;
    if (!ws || misaligned(ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    rc = view_workspace_bytes(c, op, batch, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(c, CKKS_ENOMEM, "workspace too small");
    return CKKS_OK;
}

// ModUp side shared by every key switch: w.x holds the first inverse pass of the polynomial(s).
// Second inverse pass (scaled by the conversion pre-factor), then conversion fused into the
// first forward pass of every extended limb.
static void decompose_extend(const View* c, const Workspace& w, u32 groups, hipStream_t s, bool fp_beside = false) {
    const LimbSel sel = {c->L, groups, c->L, 0, 0, 0};
    const u32 fmt = conv_on_matrix_cores(c, CONV_UP) ? SRC_DIGITS : SRC_F64;
    InvStridedArgs a2 = {w.x, sel, SC_UP, fmt};
    launch_inv_strided(c, a2, s);
    ConvArgs a3 = {w.x, w.dt, groups, fmt};
    SideStream& sd = c->sh->side;
    if (fp_beside && sd.enabled && c->mixed_classes && !sd.active && side_stream_ready(sd)) {
        // the IntAr targets first, on s; the FpAr targets on the side stream from the moment those are done, beside
        // whatever s runs next (the caller joins before it reads the FpAr limbs of dt)
        launch_conv<CONV_UP>(c, a3, s, 0);
        hipEvent_t e = side_event(sd);
        if (e && hipEventRecord(e, s) == hipSuccess && hipStreamWaitEvent(sd.stream, e, 0) == hipSuccess) {
            launch_conv<CONV_UP>(c, a3, sd.stream, 1);
            sd.fp_pending = true;
            return;
        }
        (void)hipGetLastError();
        launch_conv<CONV_UP>(c, a3, s, 1);
        return;
    }
    fork_side(c, s);  // from here the special-limb (IntAr) chain runs beside the q-limb chain
    launch_conv<CONV_UP>(c, a3, s);
}

static bool any_fp_prime(const View* c, u32 lo, u32 hi) {
    for (u32 i = lo; i < hi; i++)
        if (c->primes[i] < CKKS_FP_PRIME_LIMIT) return true;
    return false;
}

// s waits for the FpAr conversion that decompose_extend put on the side stream
static void join_fp_beside(const View* c, hipStream_t s) {
    SideStream& sd = c->sh->side;
    if (!sd.fp_pending) return;
    sd.fp_pending = false;
    hipEvent_t e = side_event(sd);
    if (!e || hipEventRecord(e, sd.stream) != hipSuccess || hipStreamWaitEvent(s, e, 0) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipStreamSynchronize(sd.stream);
    }
}

// ModDown side: w.cp holds the first inverse pass of c' on the special limbs.
static void moddown_convert(const View* c, const Workspace& w, u32 cg, hipStream_t s) {
    const LimbSel sel = {c->K, cg * 2, c->K, 0, c->L, 0};
    const u32 fmt = conv_on_matrix_cores(c, CONV_DN) ? SRC_DIGITS : SRC_CANON;
    InvStridedArgs a6 = {w.cp, sel, SC_DN, fmt};
    launch_inv_strided(c, a6, s);
    join_side(c, s);  // the conversion reads every special limb
    ConvArgs a7 = {w.cp, w.cv, cg * 2, fmt};
    launch_conv<CONV_DN>(c, a7, s);
}

// cm: the view whose ModDown ends the pipeline: c itself, or the merged view of c's level (the ModDown then
// also divides by the last q-limb: limb c->L - 1 joins the special limbs and the output has c->L - 1 limbs)
// multi_galois / multi_keys (rotations only, batch <= CKKS_ROT_CHUNK): one Galois element and key per instance.
template <int LOAD, int OWN>
static void keyswitch_pipeline(const View* c, const View* cm, const u64* in1, const u64* in2, const u64* key, u64* out,
                               u32 batch, u32 galois, void* ws, hipStream_t s, const u32* multi_galois = nullptr,
                               const u64* const* multi_keys = nullptr) {
    Workspace w = carve(c, ws, batch, batch, batch, false);
    if (cm != c)  // cv shrinks by one limb per component, cp grows by one: still inside the level's workspace
        w.cv = w.cp + ((size_t)batch * 2 * cm->K << c->logN);
    const LimbSel sel = {c->L, batch, c->L, 0, 0, 0};
    InvContigArgs a1;
    memset(&a1, 0, sizeof(a1));
    a1.src = in1, a1.src2 = in2, a1.dst = w.x, a1.sel = sel, a1.dsel = sel, a1.galois[0] = galois;
    InnerArgs ia;
    memset(&ia, 0, sizeof(ia));
    ia.key[0] = key, ia.galois[0] = galois;
    if (multi_galois) {
        a1.per_inst = ia.per_inst = 1;
        for (u32 b = 0; b < batch; b++)
            a1.galois[b] = ia.galois[b] = multi_galois[b], ia.key[b] = multi_keys[b];
    }
    launch_inv_contig<LOAD>(c, a1, s);
    decompose_extend(c, w, batch, s, true);
    ia.dt = w.dt, ia.own = in1, ia.own2 = in2;
    ia.cq = w.cq, ia.cp = w.cp, ia.n_inst = batch, ia.split = cm->L;
    // the limbs that feed the ModDown conversion first; the q-limbs then finish in one kernel, c' in registers.
    // Those of them that are FpAr primes (special primes below the FP64 limit; limb cm->L of the merged rescale) take
    // their digits from the FpAr conversion, which may still be running on the side stream.
    if (any_fp_prime(c, cm->L, c->D)) join_fp_beside(c, s);
    if (cm != c) {
        launch_ks_inner<OWN, false, false>(c, ia, s, cm->L, c->D);
    } else {
        // special limbs belong to no digit, so every variant computes the same on them: the leanest one runs
        launch_ks_inner<OWN_COPY, false, false>(c, ia, s, c->L, c->D);
    }
    moddown_convert(cm, w, batch, s);
    ia.cv = w.cv, ia.out = out, ia.fin_pinv = cm->tb.pinv;
    join_fp_beside(c, s);
    launch_ks_inner<OWN, false, true>(c, ia, s, 0, cm->L);
}

extern "C" int ckks_keyswitch_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_d, const uint64_t* d_key,
                                 uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    int rc = check_ks_args(c, d_d, d_key, d_out, batch, CKKS_OP_KEYSWITCH, d_ws, ws_bytes);
    if (rc) return rc;
    rc = check_no_alias(c, d_out, limb_bytes(c, (size_t)batch * 2 * c->L), d_d, limb_bytes(c, (size_t)batch * c->L), nullptr, 0,
                        d_ws, ws_bytes);
    if (rc) return rc;
    keyswitch_pipeline<INV_PLAIN, OWN_COPY>(c, c, d_d, nullptr, d_key, d_out, batch, 1, d_ws, (hipStream_t)stream);
    return hip_check(c, "ckks_keyswitch");
}

extern "C" int ckks_hmult_relin_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct1, const uint64_t* d_ct2,
                                   const uint64_t* d_evk, uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes,
                                   void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (!d_ct2 || misaligned(d_ct2, 16)) return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_args(c, d_ct1, d_evk, d_out, batch, CKKS_OP_HMULT_RELIN, d_ws, ws_bytes);
    if (rc) return rc;
    const size_t ctb = limb_bytes(c, (size_t)batch * 2 * c->L);
    rc = check_no_alias(c, d_out, ctb, d_ct1, ctb, d_ct2, ctb, d_ws, ws_bytes);
    if (rc) return rc;
    keyswitch_pipeline<INV_TENSOR, OWN_TENSOR>(c, c, d_ct1, d_ct2, d_evk, d_out, batch, 1, d_ws,
                                                          (hipStream_t)stream);
    return hip_check(c, "ckks_hmult_relin");
}

extern "C" int ckks_hmult_relin_rescale_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct1, const uint64_t* d_ct2,
                                           const uint64_t* d_evk, uint64_t* d_out, uint32_t batch, void* d_ws,
                                           size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (level < 2) return fail(c, CKKS_EINVAL, "rescale needs at least two limbs");
    if (!d_ct2 || misaligned(d_ct2, 16)) return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    int rc = check_ks_args(c, d_ct1, d_evk, d_out, batch, CKKS_OP_HMULT_RELIN, d_ws, ws_bytes);
    if (rc) return rc;
    const size_t ctb = limb_bytes(c, (size_t)batch * 2 * c->L);
    rc = check_no_alias(c, d_out, limb_bytes(c, (size_t)batch * 2 * (c->L - 1)), d_ct1, ctb, d_ct2, ctb, d_ws, ws_bytes);
    if (rc) return rc;
    keyswitch_pipeline<INV_TENSOR, OWN_TENSOR>(c, &ctx->merged[level], d_ct1, d_ct2, d_evk, d_out, batch, 1,
                                                             d_ws, (hipStream_t)stream);
    return hip_check(c, "ckks_hmult_relin_rescale");
}

extern "C" int ckks_hrot_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t galois, const uint64_t* d_rk,
                            uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    int rc = check_ks_args(c, d_ct, d_rk, d_out, batch, CKKS_OP_HROT, d_ws, ws_bytes);
    if (rc) return rc;
    rc = check_galois(c, galois);
    if (rc) return rc;
    const size_t ctb = limb_bytes(c, (size_t)batch * 2 * c->L);
    rc = check_no_alias(c, d_out, ctb, d_ct, ctb, nullptr, 0, d_ws, ws_bytes);
    if (rc) return rc;
    keyswitch_pipeline<INV_ROT, OWN_ROT>(c, c, d_ct, nullptr, d_rk, d_out, batch, galois, d_ws,
                                                   (hipStream_t)stream);
    return hip_check(c, "ckks_hrot");
}

extern "C" int ckks_keyswitch(ckks_ctx* ctx, const uint64_t* d_d, const uint64_t* d_key, uint64_t* d_out,
                              uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_keyswitch_at(ctx, ctx->L, d_d, d_key, d_out, batch, d_ws, ws_bytes, stream);
}

extern "C" int ckks_hmult_relin(ckks_ctx* ctx, const uint64_t* d_ct1, const uint64_t* d_ct2, const uint64_t* d_evk,
                                uint64_t* d_out, uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_hmult_relin_at(ctx, ctx->L, d_ct1, d_ct2, d_evk, d_out, batch, d_ws, ws_bytes, stream);
}

extern "C" int ckks_hrot(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t galois, const uint64_t* d_rk, uint64_t* d_out,
                         uint32_t batch, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_hrot_at(ctx, ctx->L, d_ct, galois, d_rk, d_out, batch, d_ws, ws_bytes, stream);
}

// Rescale = a ModDown whose only special prime is the last active limb: inverse transform of that
// limb, reduction modulo every remaining prime fused into their first forward pass, second forward
// pass fused with (c_i - .) * q_last^-1.
static int rescale_impl(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint64_t* d_out, uint32_t batch,
                        void* d_ws, size_t ws_bytes, void* stream, bool static_scratch) {
    if (!ctx) return CKKS_EINVAL;
    if (level < 2 || level > ctx->L) return fail(ctx, CKKS_EINVAL, "rescale needs a level between 2 and L");
    const View* c = &ctx->rescale[level];  // c->L = level - 1 targets, c->K = 1
    if (!d_ct || !d_out || misaligned(d_ct, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (batch == 0 || batch > 4096) return fail(c, CKKS_EINVAL, "batch out of range");
    if (!d_ws || misaligned(d_ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    const size_t N = (size_t)1 << c->logN;
    if (ws_bytes < (size_t)batch * 2 * level * N * sizeof(u64))
        return fail(c, CKKS_ENOMEM, static_scratch ? "batch * 2 * level * N words exceed CKKS_STATIC_SCRATCH_BYTES"
                                                   : "workspace too small");
    int rc = check_no_alias(c, d_out, limb_bytes(c, (size_t)batch * 2 * (level - 1)), d_ct, limb_bytes(c, (size_t)batch * 2 * level),
                            nullptr, 0, d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    Workspace w;
    w.x = w.dt = w.cq = nullptr;
    w.cp = (u64*)d_ws;                    // [b][2][1][N]
    w.cv = w.cp + (size_t)batch * 2 * N;  // [b][2][level-1][N]
    const LimbSel src = {1, batch * 2, level, level - 1, level - 1, 0};  // limb level-1 of every component
    const LimbSel dst = {1, batch * 2, 1, 0, level - 1, 0};
    InvContigArgs a1 = {d_ct, nullptr, w.cp, src, dst, {1}, 0};
    launch_inv_contig<INV_PLAIN>(c, a1, s);
    moddown_convert(c, w, batch, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cq = d_ct, fa.cq_L = level, fa.cv = w.cv, fa.out = d_out, fa.n_inst = batch;
    launch_ks_final<FIN_KS>(c, fa, s);
    return hip_check(c, "ckks_rescale");
}

extern "C" int ckks_rescale(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint64_t* d_out, uint32_t batch,
                            void* d_ws, size_t ws_bytes, void* stream) {
    return rescale_impl(ctx, level, d_ct, d_out, batch, d_ws, ws_bytes, stream, false);
}

// The same launches with the workspace in this GPU's static scratch array: no allocation of any kind, no
// workspace argument.  Every word of the scratch that the kernels read has been written earlier in the same
// call (last-limb coefficients, then the converted part), so nothing has to be cleared between calls.
extern "C" int ckks_rescale_static(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint64_t* d_out, uint32_t batch,
                                   void* stream) {
    if (!ctx) return CKKS_EINVAL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, CKKS_EINVAL, "the current device is not the one the context was created on");
    return rescale_impl(ctx, level, d_ct, d_out, batch, ctx->scratch_ptr, CKKS_STATIC_SCRATCH_BYTES, stream, true);
}

extern "C" int ckks_hrot_hoisted_mac_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot,
                                        const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt,
                                        uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (!h_galois || !h_rk_ptrs) return fail(c, CKKS_EINVAL, "null host array");
    if (n_rot == 0 || n_rot > 65535) return fail(c, CKKS_EINVAL, "n_rot out of range");
    if (!d_ct || !d_pt || !d_out || misaligned(d_ct, 16) || misaligned(d_pt, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (!d_ws || misaligned(d_ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    int rc = view_workspace_bytes(c, CKKS_OP_HROT_HOISTED_MAC, n_rot, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(c, CKKS_ENOMEM, "workspace too small");
    for (u32 r = 0; r < n_rot; r++) {
        if (!h_rk_ptrs[r] || misaligned(h_rk_ptrs[r], 16)) return fail(c, CKKS_EINVAL, "null or misaligned key");
        rc = check_galois(c, h_galois[r]);
        if (rc) return rc;
    }
    rc = check_no_alias(c, d_out, limb_bytes(c, 2 * (size_t)c->L), d_ct, limb_bytes(c, 2 * (size_t)c->L), d_pt,
                        limb_bytes(c, (size_t)n_rot * c->L), d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const size_t N = (size_t)1 << c->logN;
    const u32 chunk_max = n_rot < CKKS_ROT_CHUNK ? n_rot : CKKS_ROT_CHUNK;
    const Workspace w = carve(c, d_ws, 1, 1, chunk_max);
    // hoisted part: decompose a = ct[1] once and finish the transform of every extended limb
    {
        const LimbSel src = {c->L, 1, c->L, c->L, 0, 0};  // limbs L .. 2L-1 of ct, primes 0 .. L-1
        const LimbSel dst = {c->L, 1, c->L, 0, 0, 0};
        InvContigArgs a1 = {d_ct, nullptr, w.x, src, dst, {1}, 0};
        launch_inv_contig<INV_PLAIN>(c, a1, s);
        decompose_extend(c, w, 1, s);
        if (c->dnum > 1) {
            FwdContigArgs q = {w.dt, LimbSel{c->L, c->dnum - 1, c->D, 0, 0, c->alpha}};
            launch_fwd_contig(c, q, s);
        }
        FwdContigArgs p = {w.dt, LimbSel{c->K, c->dnum, c->D, c->L, c->L, 0}};
        launch_fwd_contig(c, p, s);
    }
    // rotations go through the ModDown side in chunks of at most CKKS_ROT_CHUNK, sized evenly
    const u32 n_chunks = (n_rot + CKKS_ROT_CHUNK - 1) / CKKS_ROT_CHUNK;
    const u32 chunk = (n_rot + n_chunks - 1) / n_chunks;
    for (u32 r0 = 0; r0 < n_rot; r0 += chunk) {
        const u32 nr = (n_rot - r0) < chunk ? (n_rot - r0) : chunk;
        InnerArgs ia;
        memset(&ia, 0, sizeof(ia));
        FinalArgs fa;
        memset(&fa, 0, sizeof(fa));
        for (u32 r = 0; r < nr; r++) {
            ia.key[r] = h_rk_ptrs[r0 + r];
            ia.galois[r] = h_galois[r0 + r];
            fa.galois[r] = h_galois[r0 + r];
        }
        ia.dt = w.dt, ia.own = d_ct, ia.cq = w.cq, ia.cp = w.cp, ia.n_inst = nr, ia.split = c->L;
        fork_side(c, s);  // no-op in the first chunk (still forked); later chunks wait for the previous ModDown
        launch_ks_inner<OWN_COPY, true>(c, ia, s);
        moddown_convert(c, w, nr, s);
        fa.cq = w.cq, fa.cq_L = c->L, fa.cv = w.cv, fa.ct1 = d_ct, fa.pt = d_pt + (size_t)r0 * c->L * N, fa.out = d_out;
        fa.n_inst = 2, fa.n_rot = nr, fa.accumulate = r0 ? 1 : 0;
        launch_ks_final<FIN_HOISTED>(c, fa, s);
    }
    return hip_check(c, "ckks_hrot_hoisted_mac");
}

extern "C" int ckks_hrot_hoisted_mac(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                                     const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out,
                                     void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_hrot_hoisted_mac_at(ctx, ctx->L, d_ct, n_rot, h_galois, h_rk_ptrs, d_pt, d_out, d_ws, ws_bytes, stream);
}

// Double-hoisted variant: the plaintext products are accumulated in the extended basis over all
// rotations (CKKS_DH_CHUNK of them per launch) and a single ModDown follows.
static int dh_mac_impl(ckks_ctx* ctx, uint32_t level, bool rescale, const uint64_t* d_ct, uint32_t n_rot,
                       const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt,
                       uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (rescale && level < 2) return fail(c, CKKS_EINVAL, "rescale needs at least two limbs");
    if (!h_galois || !h_rk_ptrs) return fail(c, CKKS_EINVAL, "null host array");
    if (n_rot == 0 || n_rot > 65535) return fail(c, CKKS_EINVAL, "n_rot out of range");
    if (!d_ct || !d_pt || !d_out || misaligned(d_ct, 16) || misaligned(d_pt, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (!d_ws || misaligned(d_ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    int rc = view_workspace_bytes(c, CKKS_OP_HROT_DH_MAC, n_rot, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(c, CKKS_ENOMEM, "workspace too small");
    for (u32 r = 0; r < n_rot; r++) {
        if (!h_rk_ptrs[r] || misaligned(h_rk_ptrs[r], 16)) return fail(c, CKKS_EINVAL, "null or misaligned key");
        rc = check_galois(c, h_galois[r]);
        if (rc) return rc;
    }
    rc = check_no_alias(c, d_out, limb_bytes(c, 2 * (size_t)(rescale ? c->L - 1 : c->L)), d_ct, limb_bytes(c, 2 * (size_t)c->L),
                        d_pt, limb_bytes(c, (size_t)n_rot * c->D), d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const size_t N = (size_t)1 << c->logN;
    // cm: the view whose ModDown ends the call (the merged one also divides by the last q-limb)
    const View* cm = rescale ? &ctx->merged[level] : c;
    Workspace w = carve(c, d_ws, 1, 1, 1);
    if (rescale) {
        w.cp = w.cq + (size_t)2 * cm->L * N;
        w.cv = w.cp + (size_t)2 * cm->K * N;
    }
    {  // hoisted part, as in ckks_hrot_hoisted_mac
        const LimbSel src = {c->L, 1, c->L, c->L, 0, 0};
        const LimbSel dst = {c->L, 1, c->L, 0, 0, 0};
        InvContigArgs a1 = {d_ct, nullptr, w.x, src, dst, {1}, 0};
        launch_inv_contig<INV_PLAIN>(c, a1, s);
        decompose_extend(c, w, 1, s);
        if (c->dnum > 1) {
            FwdContigArgs q = {w.dt, LimbSel{c->L, c->dnum - 1, c->D, 0, 0, c->alpha}};
            launch_fwd_contig(c, q, s);
        }
        FwdContigArgs p = {w.dt, LimbSel{c->K, c->dnum, c->D, c->L, c->L, 0}};
        launch_fwd_contig(c, p, s);
    }
    // the special-limb chain (still on the side stream when overlap is on) only reads its own limbs
    for (u32 r0 = 0; r0 < n_rot; r0 += CKKS_DH_CHUNK) {
        const u32 nr = (n_rot - r0) < CKKS_DH_CHUNK ? (n_rot - r0) : CKKS_DH_CHUNK;
        DhInnerArgs ia;
        memset(&ia, 0, sizeof(ia));
        for (u32 r = 0; r < nr; r++) ia.key[r] = h_rk_ptrs[r0 + r], ia.galois[r] = h_galois[r0 + r];
        ia.dt = w.dt, ia.ct = d_ct, ia.pt = d_pt + (size_t)r0 * c->D * N, ia.cq = w.cq, ia.cp = w.cp;
        ia.n_rot = nr, ia.accumulate = r0 ? 1 : 0, ia.split = cm->L;
        launch_dh_accum(c, ia, s);
    }
    {  // ModDown of the sum: first inverse pass of its source limbs, then the shared tail
        const LimbSel sel = {cm->K, 2, cm->K, 0, cm->L, 0};
        InvContigArgs ic = {w.cp, nullptr, w.cp, sel, sel, {1}, 0};
        launch_inv_contig<INV_PLAIN>(cm, ic, s);
    }
    moddown_convert(cm, w, 1, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cq = w.cq, fa.cq_L = cm->L, fa.cv = w.cv, fa.out = d_out, fa.n_inst = 1;
    launch_ks_final<FIN_KS>(cm, fa, s);
    return hip_check(c, "ckks_hrot_dh_mac");
}

extern "C" int ckks_hrot_dh_mac_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot,
                                   const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt,
                                   uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    return dh_mac_impl(ctx, level, false, d_ct, n_rot, h_galois, h_rk_ptrs, d_pt, d_out, d_ws, ws_bytes, stream);
}

extern "C" int ckks_hrot_dh_mac_rescale_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n_rot,
                                           const uint32_t* h_galois, const uint64_t* const* h_rk_ptrs,
                                           const uint64_t* d_pt, uint64_t* d_out, void* d_ws, size_t ws_bytes,
                                           void* stream) {
    return dh_mac_impl(ctx, level, true, d_ct, n_rot, h_galois, h_rk_ptrs, d_pt, d_out, d_ws, ws_bytes, stream);
}

extern "C" int ckks_hrot_dh_mac(ckks_ctx* ctx, const uint64_t* d_ct, uint32_t n_rot, const uint32_t* h_galois,
                                const uint64_t* const* h_rk_ptrs, const uint64_t* d_pt, uint64_t* d_out, void* d_ws,
                                size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    return ckks_hrot_dh_mac_at(ctx, ctx->L, d_ct, n_rot, h_galois, h_rk_ptrs, d_pt, d_out, d_ws, ws_bytes, stream);
}

// ---------------------------------------------------------------- baby-step giant-step transform
static size_t bsgs_workspace_words(const View* c, u32 n1, u32 n2) {
    const size_t N = (size_t)1 << c->logN;
    const u32 nc = n2 < CKKS_ROT_CHUNK ? n2 : CKKS_ROT_CHUNK;
    const size_t limbs = (size_t)c->L + (size_t)c->dnum * c->D                      // x, dt of the input
                         + (size_t)n1 * 2 * c->D                                     // baby rotations, extended basis
                         + (size_t)n2 * 2 * (2 * (size_t)c->L + c->K)                // C on q / special limbs, converted part
                         + (size_t)n2 * 2 * c->L * 2;                                // inner sums, rotated inner sums
    return limbs * N + ks_workspace_words(c, nc, nc, nc, false);  // the giant rotations run the plain pipeline
}

extern "C" int ckks_lintrans_bsgs_workspace_bytes(const ckks_ctx* ctx, uint32_t level, uint32_t n1, uint32_t n2,
                                                  size_t* bytes) {
    if (!ctx || !bytes) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (c->K == 0) return fail(c, CKKS_EUNSUPPORTED, "context has no special primes");
    if (n1 == 0 || n1 > 64 || n2 == 0 || n2 > 64) return fail(c, CKKS_EINVAL, "n1 and n2 must be between 1 and 64");
    *bytes = bsgs_workspace_words(c, n1, n2) * sizeof(u64);
    return CKKS_OK;
}

extern "C" int ckks_lintrans_bsgs_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, uint32_t n1,
                                     const uint32_t* h_baby_galois, const uint64_t* const* h_baby_rk_ptrs, uint32_t n2,
                                     const uint32_t* h_giant_galois, const uint64_t* const* h_giant_rk_ptrs,
                                     const uint64_t* d_pt, uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (!h_baby_galois || !h_baby_rk_ptrs || !h_giant_galois || !h_giant_rk_ptrs) return fail(c, CKKS_EINVAL, "null host array");
    if (!d_ct || !d_pt || !d_out || misaligned(d_ct, 16) || misaligned(d_pt, 16) || misaligned(d_out, 16))
        return fail(c, CKKS_EINVAL, "null or misaligned buffer");
    if (!d_ws || misaligned(d_ws, 256)) return fail(c, CKKS_EINVAL, "workspace is null or not 256-byte aligned");
    size_t need = 0;
    int rc = ckks_lintrans_bsgs_workspace_bytes(ctx, level, n1, n2, &need);
    if (rc) return rc;
    if (ws_bytes < need) return fail(c, CKKS_ENOMEM, "workspace too small");
    for (u32 r = 0; r < n1 + n2; r++) {
        const uint64_t* k = r < n1 ? h_baby_rk_ptrs[r] : h_giant_rk_ptrs[r - n1];
        if (!k || misaligned(k, 16)) return fail(c, CKKS_EINVAL, "null or misaligned key");
        rc = check_galois(c, r < n1 ? h_baby_galois[r] : h_giant_galois[r - n1]);
        if (rc) return rc;
    }
    rc = check_no_alias(c, d_out, limb_bytes(c, 2 * (size_t)c->L), d_ct, limb_bytes(c, 2 * (size_t)c->L), d_pt,
                        limb_bytes(c, (size_t)n1 * n2 * c->D), d_ws, ws_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const size_t N = (size_t)1 << c->logN, LN = (size_t)c->L * N, KN = (size_t)c->K * N;
    // workspace: x | dt | Rq | Rp | Cq | Cp | Cv | inner | rot | key-switch workspace of the giant rotations
    Workspace w;
    w.x = (u64*)d_ws;
    w.dt = w.x + LN;
    u64* rq = w.dt + (size_t)c->dnum * c->D * N;
    u64* rp = rq + (size_t)n1 * 2 * LN;
    w.cq = rp + (size_t)n1 * 2 * KN;
    w.cp = w.cq + (size_t)n2 * 2 * LN;
    w.cv = w.cp + (size_t)n2 * 2 * KN;
    u64* inner = w.cv + (size_t)n2 * 2 * LN;
    u64* rot = inner + (size_t)n2 * 2 * LN;
    void* ks_ws = rot + (size_t)n2 * 2 * LN;
    {  // decomposition of the input, shared by every baby step
        const LimbSel src = {c->L, 1, c->L, c->L, 0, 0};
        const LimbSel dst = {c->L, 1, c->L, 0, 0, 0};
        InvContigArgs a1 = {d_ct, nullptr, w.x, src, dst, {1}, 0};
        launch_inv_contig<INV_PLAIN>(c, a1, s);
        decompose_extend(c, w, 1, s);
        if (c->dnum > 1) {
            FwdContigArgs q = {w.dt, LimbSel{c->L, c->dnum - 1, c->D, 0, 0, c->alpha}};
            launch_fwd_contig(c, q, s);
        }
        FwdContigArgs p = {w.dt, LimbSel{c->K, c->dnum, c->D, c->L, c->L, 0}};
        launch_fwd_contig(c, p, s);
    }
    // baby steps: R_b = P * Rot_b(ct) in the extended basis (inner product with the key, plus P * sigma_b(b))
    for (u32 b = 0; b < n1; b++) {
        DhInnerArgs ia;
        memset(&ia, 0, sizeof(ia));
        ia.key[0] = h_baby_rk_ptrs[b], ia.galois[0] = h_baby_galois[b];
        ia.dt = w.dt, ia.ct = d_ct, ia.pt = nullptr, ia.cq = rq + (size_t)b * 2 * LN, ia.cp = rp + (size_t)b * 2 * KN;
        ia.n_rot = 1, ia.accumulate = 0, ia.split = c->L;
        launch_dh_accum(c, ia, s);
    }
    // giant-step combinations in the extended basis, then one ModDown per giant step (as a batch)
    BsgsMacArgs ma = {rq, rp, d_pt, w.cq, w.cp, n1, n2};
    launch_bsgs_mac(c, ma, s);
    {
        const LimbSel sel = {c->K, n2 * 2, c->K, 0, c->L, 0};
        InvContigArgs ic = {w.cp, nullptr, w.cp, sel, sel, {1}, 0};
        launch_inv_contig<INV_PLAIN>(c, ic, s);
    }
    moddown_convert(c, w, n2, s);
    FinalArgs fa;
    memset(&fa, 0, sizeof(fa));
    fa.cq = w.cq, fa.cq_L = c->L, fa.cv = w.cv, fa.out = inner, fa.n_inst = n2;
    launch_ks_final<FIN_KS>(c, fa, s);
    // giant rotations, each inner sum with its own key, then the sum
    for (u32 g0 = 0; g0 < n2; g0 += CKKS_ROT_CHUNK) {
        const u32 ng = (n2 - g0) < CKKS_ROT_CHUNK ? (n2 - g0) : CKKS_ROT_CHUNK;
        keyswitch_pipeline<INV_ROT, OWN_ROT>(c, c, inner + (size_t)g0 * 2 * LN, nullptr, nullptr,
                                                       rot + (size_t)g0 * 2 * LN, ng, 1, ks_ws, s, h_giant_galois + g0,
                                                       h_giant_rk_ptrs + g0);
    }
    {
        ProfScope ps(c, std::string("sum_instances_kernel"), (u64)(n2 + 1) * 2 * c->L, s);
        hipLaunchKernelGGL(sum_instances_kernel, dim3((1u << c->logN) / 256, 2 * c->L), dim3(256), 0, s, rot, d_out,
                           c->tb.pc, c->logN, c->L, 2 * c->L, n2);
    }
    return hip_check(c, "ckks_lintrans_bsgs");
}

// Rotations of a batch of ciphertexts, each by its own Galois element with its own key (the giant steps of a
// linear transform, or the independent rotations of several activations): chunks of CKKS_ROT_CHUNK instances.
extern "C" int ckks_hrot_multi_at(ckks_ctx* ctx, uint32_t level, const uint64_t* d_ct, const uint32_t* h_galois,
                                  const uint64_t* const* h_rk_ptrs, uint64_t* d_out, uint32_t batch, void* d_ws,
                                  size_t ws_bytes, void* stream) {
    if (!ctx) return CKKS_EINVAL;
    const View* c = view_at(ctx, level);
    if (!c) return CKKS_EINVAL;
    if (!h_galois || !h_rk_ptrs) return fail(c, CKKS_EINVAL, "null host array");
    if (batch == 0) return fail(c, CKKS_EINVAL, "batch out of range");
    const u32 chunk = batch < CKKS_ROT_CHUNK ? batch : CKKS_ROT_CHUNK;
    int rc = check_ks_args(c, d_ct, h_rk_ptrs[0], d_out, chunk, CKKS_OP_HROT, d_ws, ws_bytes);
    if (rc) return rc;
    if (batch > 4096) return fail(c, CKKS_EINVAL, "batch out of range");
    for (u32 b = 0; b < batch; b++) {
        if (!h_rk_ptrs[b] || misaligned(h_rk_ptrs[b], 16)) return fail(c, CKKS_EINVAL, "null or misaligned key");
        rc = check_galois(c, h_galois[b]);
        if (rc) return rc;
    }
    const size_t ct_words = ((size_t)2 * c->L) << c->logN;
    rc = check_no_alias(c, d_out, ct_words * batch * sizeof(u64), d_ct, ct_words * batch * sizeof(u64), nullptr, 0, d_ws, ws_bytes);
    if (rc) return rc;
    for (u32 b0 = 0; b0 < batch; b0 += CKKS_ROT_CHUNK) {
        const u32 nb = (batch - b0) < CKKS_ROT_CHUNK ? (batch - b0) : CKKS_ROT_CHUNK;
        keyswitch_pipeline<INV_ROT, OWN_ROT>(c, c, d_ct + b0 * ct_words, nullptr, nullptr, d_out + b0 * ct_words, nb,
                                                       1, d_ws, (hipStream_t)stream, h_galois + b0, h_rk_ptrs + b0);
    }
    return hip_check(c, "ckks_hrot_multi");
}
