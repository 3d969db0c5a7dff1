// Host side of the context: prime chain, roots of unity, NTT twiddle tables, base-conversion
// tables, Montgomery constants, the canonical-embedding FFT used by encode/decode.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <complex>

#include "common.h"

void cm_ops_forget_ctx(cm_ctx *ctx);
void cm_ops_device_init();
static thread_local int g_hip_error = 0;
void cm_set_hip_error(int e) { g_hip_error = e; }
extern "C" int32_t cm_last_hip_error(void) { return g_hip_error; }
extern "C" const char *cm_strerror(cm_status s) {
    switch (s) {
        case CM_OK: return "ok";
        case CM_E_INVAL: return "invalid argument";
        case CM_E_LEVEL: return "level exhausted or level mismatch";
        case CM_E_SCALE: return "scale mismatch";
        case CM_E_NOKEY: return "evaluation key for this rotation step / relinearisation not generated";
        case CM_E_LAYOUT: return "plan, cache and ciphertext shapes do not fit together";
        case CM_E_NOMEM: return "out of memory";
        case CM_E_HIP: return "HIP runtime error (see cm_last_hip_error)";
        case CM_E_TOOBIG: return "operand larger than the fixed work area of this entry point";
    }
    return "unknown status";
}

// ---- kernel-family timing ---------------------------------------------------------------------------
Prof::Prof(cm_ctx *ctx, int fam, double units, hipStream_t s) : c(ctx), st(s), e0(0), live(ctx->prof.on) {
    if (!live) return;
    ProfState &p = c->prof;
    e0 = 2 * p.recs.size();
    while (p.pool.size() < e0 + 2) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { live = false; return; }
        p.pool.push_back(e);
    }
    p.recs.push_back({fam, units, e0});
    hipEventRecord(p.pool[e0], st);
}
Prof::~Prof() {
    if (live) hipEventRecord(c->prof.pool[e0 + 1], st);
}
extern "C" cm_status cm_profile_enable(cm_ctx *ctx, int32_t on) {
    if (!ctx) return CM_E_INVAL;
    ctx->prof.on = on != 0;
    ctx->prof.recs.clear();
    return CM_OK;
}
extern "C" cm_status cm_ctx_set_option(cm_ctx *ctx, int32_t option, int32_t value) {
    if (!ctx) return CM_E_INVAL;
    switch (option) {
        case CM_OPT_EVK_STORED_A: ctx->evk_stored_a = value != 0; return CM_OK;
        case CM_OPT_TWO_STEP_MASKS: ctx->two_step_masks = value != 0; return CM_OK;
    }
    return CM_E_INVAL;
}
extern "C" cm_status cm_profile_get(cm_ctx *ctx, int32_t family, double *launches, double *units, double *ms) {
    if (!ctx || family < 0 || family >= CM_K_FAMILIES) return CM_E_INVAL;
    double l = 0, u = 0, t = 0;
    for (auto &r : ctx->prof.recs) {
        if (r.fam != family) continue;
        float dt = 0;
        HIPCHK(hipEventSynchronize(ctx->prof.pool[r.e0 + 1]));
        HIPCHK(hipEventElapsedTime(&dt, ctx->prof.pool[r.e0], ctx->prof.pool[r.e0 + 1]));
        l += 1, u += r.units, t += dt;
    }
    if (launches) *launches = l;
    if (units) *units = u;
    if (ms) *ms = t;
    return CM_OK;
}

// ---- number theory on the host -----------------------------------------------------------------
u64 h_mulmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a * b) % q); }
u64 h_powmod(u64 b, u64 e, u64 q) {
    u64 r = 1 % q;
    b %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = h_mulmod(r, b, q);
        b = h_mulmod(b, b, q);
    }
    return r;
}
u64 h_invmod(u64 a, u64 q) { return h_powmod(a % q, q - 2, q); }   // q prime
u64 h_shoup(u64 w, u64 q) { return (u64)((((u128)w) << 64) / q); }

static bool h_is_prime(u64 m) {
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (m < 2) return false;
    for (u64 b : bases)
        if (m % b == 0) return m == b;
    u64 d = m - 1;
    int r = 0;
    while (!(d & 1)) d >>= 1, r++;
    for (u64 a : bases) {
        u64 x = h_powmod(a, d, m);
        if (x == 1 || x == m - 1) continue;
        bool comp = true;
        for (int i = 1; i < r && comp; i++) {
            x = h_mulmod(x, x, m);
            if (x == m - 1) comp = false;
        }
        if (comp) return false;
    }
    return true;
}
// primes among 2^bits + 1 - k*2n, k = 1, 2, ..., in that order
static std::vector<u64> scan_primes(int bits, int n, int count) {
    std::vector<u64> out;
    for (u64 k = 1; (int)out.size() < count; k++) {
        u64 c = (1ULL << bits) + 1 - k * 2 * (u64)n;
        if (h_is_prime(c)) out.push_back(c);
    }
    return out;
}
static u64 root_2n(u64 q, int n) {
    for (u64 x = 2;; x++) {
        u64 psi = h_powmod(x, (q - 1) / (2 * (u64)n), q);
        if (h_powmod(psi, (u64)n, q) == q - 1) return psi;
    }
}
static u64 brev(u64 x, int bits) {
    u64 r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}

u64 galois_of_step(const cm_ctx *ctx, int step) {
    int S = ctx->n / 2;
    int r = ((step % S) + S) % S;
    return h_powmod(5, (u64)r, 2 * (u64)ctx->n);
}

std::vector<std::vector<int>> digits_at(const cm_ctx *ctx, int level) {
    std::vector<std::vector<int>> out;
    for (int s = 0; s <= level; s += ctx->alpha) {
        std::vector<int> D;
        for (int i = s; i < s + ctx->alpha && i <= level; i++) D.push_back(i);
        out.push_back(D);
    }
    return out;
}

// device copy of a host table; a failed allocation or copy raises std::bad_alloc (caught at the C boundary)
template <class T>
static T *upload(const std::vector<T> &v) {
    T *d = nullptr;
    if (hipMalloc((void **)&d, v.size() * sizeof(T)) != hipSuccess) throw std::bad_alloc();
    if (hipMemcpy(d, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) {
        hipFree(d);
        throw std::bad_alloc();
    }
    return d;
}

// Fast base conversion tables src -> dst:  hat_m = prod(src)/q_m.
static ConvTable make_conv(cm_ctx *ctx, const std::vector<int> &src, const std::vector<int> &dst) {
    ConvTable t;
    t.ns = (int)src.size();
    t.nt = (int)dst.size();
    t.src = src;
    t.dst = dst;
    std::vector<u64> inv_hat(t.ns), inv_hat_sh(t.ns), hat_mont((size_t)t.ns * t.nt);
    for (int m = 0; m < t.ns; m++) {
        u64 qm = ctx->mod[src[m]];
        u64 h = 1;
        for (int o = 0; o < t.ns; o++)
            if (o != m) h = h_mulmod(h, ctx->mod[src[o]] % qm, qm);
        inv_hat[m] = h_invmod(h, qm);
        inv_hat_sh[m] = h_shoup(inv_hat[m], qm);
        for (int r = 0; r < t.nt; r++) {
            u64 qr = ctx->mod[dst[r]];
            u64 hr = 1;
            for (int o = 0; o < t.ns; o++)
                if (o != m) hr = h_mulmod(hr, ctx->mod[src[o]] % qr, qr);
            hat_mont[(size_t)m * t.nt + r] = (u64)((((u128)hr) << 64) % qr);
        }
    }
    t.inv_hat = inv_hat;
    t.inv_hat_sh = inv_hat_sh;
    t.hat_mont = hat_mont;
    return t;
}
static void free_conv(ConvTable &) {}

const std::vector<ConvTable> &get_modup(cm_ctx *ctx, int level) {
    auto it = ctx->modup.find(level);
    if (it != ctx->modup.end()) return it->second;
    std::vector<ConvTable> tabs;
    for (auto &D : digits_at(ctx, level)) {
        std::vector<int> others;
        for (int i = 0; i <= level; i++)
            if (i < D.front() || i > D.back()) others.push_back(i);
        for (int k = 0; k < ctx->K; k++) others.push_back(ctx->L + 1 + k);
        tabs.push_back(make_conv(ctx, D, others));
    }
    return ctx->modup[level] = tabs;
}
const ConvTable &get_moddown(cm_ctx *ctx, int level) {
    auto it = ctx->moddown.find(level);
    if (it != ctx->moddown.end()) return it->second;
    std::vector<int> src, dst;
    for (int k = 0; k < ctx->K; k++) src.push_back(ctx->L + 1 + k);
    for (int i = 0; i <= level; i++) dst.push_back(i);
    return ctx->moddown[level] = make_conv(ctx, src, dst);
}
const u64 *get_pinv(cm_ctx *ctx, int level) {
    auto it = ctx->pinv.find(level);
    if (it != ctx->pinv.end()) return it->second;
    std::vector<u64> v;
    for (int i = 0; i <= level; i++) {
        u64 q = ctx->mod[i], P = 1;
        for (int k = 0; k < ctx->K; k++) P = h_mulmod(P, ctx->mod[ctx->L + 1 + k] % q, q);
        u64 inv = h_invmod(P, q);
        v.push_back(inv);
        v.push_back(h_shoup(inv, q));
    }
    return ctx->pinv[level] = upload(v);
}
const u64 *get_qlinv(cm_ctx *ctx, int level) {
    auto it = ctx->qlinv.find(level);
    if (it != ctx->qlinv.end()) return it->second;
    std::vector<u64> v;
    for (int i = 0; i < level; i++) {
        u64 q = ctx->mod[i];
        u64 inv = h_invmod(ctx->mod[level] % q, q);
        v.push_back(inv);
        v.push_back(h_shoup(inv, q));
    }
    if (v.empty()) v.push_back(0);
    return ctx->qlinv[level] = upload(v);
}

const int *iota_idx(cm_ctx *ctx) { return ctx->d_idx; }

// Cumulative table of |X| for the discrete Gaussian with sigma = 3.2 cut at 19:
// floor(2^63 * sum_{j<=k} P(j)), P(0) = w_0/Z, P(j) = 2 w_j/Z, w_j = exp(-j^2 / (2 * 3.2^2)).
static const u64 kGaussCdt[CM_GAUSS_K] = {
    0x0FF52B40A5917F1DULL, 0x2E5A25D4BF0E400EULL, 0x489AE26955B04BD6ULL, 0x5D2BC20F621BF185ULL,
    0x6BC8694C3CC80FF4ULL, 0x7532D89AC6BA7DCEULL, 0x7AB396CB74436798ULL, 0x7D9E4E916643EB07ULL,
    0x7F05495819EB2051ULL, 0x7FA1CE9C0039A957ULL, 0x7FDFB3F212E8C4E8ULL, 0x7FF5E6F9D2314FCCULL,
    0x7FFD1F97BC4406A2ULL, 0x7FFF40FA0088D11DULL, 0x7FFFD2E835E1C57DULL, 0x7FFFF6524386FF1EULL,
    0x7FFFFE1DB4769DA5ULL, 0x7FFFFFAC0A1DCB08ULL, 0x7FFFFFF428673853ULL};

extern "C" cm_status cm_ctx_create(const cm_params *p, cm_ctx **out) {
    if (!p || !out) return CM_E_INVAL;
    if (p->n != 4096 && p->n != 65536) return CM_E_INVAL;
    if (p->n_q < 1 || p->n_p < 1 || p->alpha < 1 || p->n_q + p->n_p > CM_MAX_LIMBS) return CM_E_INVAL;
    if ((p->n_q + p->alpha - 1) / p->alpha > CM_MAX_DIGITS) return CM_E_INVAL;
    if (p->alpha > CONV_MAX_SRC || p->n_p > CONV_MAX_SRC) return CM_E_INVAL;   // sources of one base conversion
    if (p->q0_bits > 61 || p->qi_bits > 61 || p->p_bits > 61 || p->q0_bits < 20 || p->qi_bits < 20 ||
        p->p_bits < 20)
        return CM_E_INVAL;
    if (fabs(p->sigma - 3.2) > 1e-12 || p->hamming < 0 || p->hamming > p->n || !(p->scale > 1)) return CM_E_INVAL;
    cm_ctx *ctx = new (std::nothrow) cm_ctx();
    if (!ctx) return CM_E_NOMEM;
    try {
    ctx->prm = *p;
    ctx->n = p->n;
    ctx->logn = p->n == 4096 ? 12 : 16;
    ctx->L = p->n_q - 1;
    ctx->K = p->n_p;
    ctx->alpha = p->alpha;
    ctx->nmod = p->n_q + p->n_p;
    const int n = ctx->n;
    if (p->q0_bits == p->qi_bits) {
        ctx->mod = scan_primes(p->qi_bits, n, p->n_q);
    } else {
        ctx->mod = scan_primes(p->q0_bits, n, 1);
        auto rest = scan_primes(p->qi_bits, n, p->n_q - 1);
        ctx->mod.insert(ctx->mod.end(), rest.begin(), rest.end());
    }
    {
        // special primes: skip any that already sit in the ciphertext chain
        std::vector<u64> sp;
        for (u64 k = 1; (int)sp.size() < p->n_p; k++) {
            u64 c = (1ULL << p->p_bits) + 1 - k * 2 * (u64)n;
            if (!h_is_prime(c)) continue;
            bool dup = false;
            for (u64 m : ctx->mod) dup |= (m == c);
            if (!dup) sp.push_back(c);
        }
        ctx->mod.insert(ctx->mod.end(), sp.begin(), sp.end());
    }
    u64 qmax = 0;
    for (u64 m : ctx->mod) qmax = m > qmax ? m : qmax;
    ctx->lazy_terms = (int)((((u128)1) << 64) / qmax) - 1;
    if (ctx->lazy_terms > 64) ctx->lazy_terms = 64;
    if (ctx->lazy_terms < 2) { delete ctx; return CM_E_INVAL; }

    // Montgomery constants and NTT tables
    std::vector<u64> tw((size_t)ctx->nmod * n), twp(tw.size()), itw(tw.size()), itwp(tw.size());
    std::vector<u64> ninv(ctx->nmod), ninvp(ctx->nmod);
    ctx->modc.resize(ctx->nmod);
    ctx->psi.resize(ctx->nmod);
    for (int m = 0; m < ctx->nmod; m++) {
        u64 q = ctx->mod[m];
        u64 inv = q;                                   // Newton: inv = q^{-1} mod 2^64
        for (int i = 0; i < 6; i++) inv *= 2 - q * inv;
        u64 r = (u64)((((u128)1) << 64) % q);
        ctx->modc[m] = ModC{q, inv, h_mulmod(r, r, q)};
        u64 psi = root_2n(q, n), psi_inv = h_invmod(psi, q);
        ctx->psi[m] = psi;
        std::vector<u64> pw(n), ipw(n);
        pw[0] = ipw[0] = 1;
        for (int i = 1; i < n; i++) {
            pw[i] = h_mulmod(pw[i - 1], psi, q);
            ipw[i] = h_mulmod(ipw[i - 1], psi_inv, q);
        }
        for (int i = 0; i < n; i++) {
            u64 e = brev((u64)i, ctx->logn);
            size_t o = (size_t)m * n + i;
            tw[o] = pw[e];
            twp[o] = h_shoup(pw[e], q);
            itw[o] = ipw[e];
            itwp[o] = h_shoup(ipw[e], q);
        }
        ninv[m] = h_invmod((u64)n, q);
        ninvp[m] = h_shoup(ninv[m], q);
    }
    ctx->d_modc = upload(ctx->modc);
    {
        std::vector<u64> pm;
        for (int i = 0; i <= ctx->L; i++) {
            u64 q = ctx->mod[i], P = 1;
            for (int k = 0; k < ctx->K; k++) P = h_mulmod(P, ctx->mod[ctx->L + 1 + k] % q, q);
            pm.push_back((u64)((((u128)P) << 64) % q));
        }
        ctx->d_pmont = upload(pm);
        std::vector<u64> ub;
        for (int i = 0; i < ctx->nmod; i++) ub.push_back(ctx->mod[i] * (0xFFFFFFFFFFFFFFFFULL / ctx->mod[i]));
        ctx->d_ubound = upload(ub);
    }
    ctx->d_tw = upload(tw);
    ctx->d_twp = upload(twp);
    ctx->d_itw = upload(itw);
    ctx->d_itwp = upload(itwp);
    ctx->d_ninv = upload(ninv);
    ctx->d_ninvp = upload(ninvp);
    {
        // double-precision copies for the FP64 butterflies: w and the correctly rounded w/q
        std::vector<double> twd(tw.size(), 0.0), twqd(tw.size(), 0.0), itwd(tw.size(), 0.0), itwqd(tw.size(), 0.0);
        std::vector<double> nd(ctx->nmod, 0.0), nqd(ctx->nmod, 0.0);
        std::vector<FpQ> fpq(ctx->nmod);
        for (int m = 0; m < ctx->nmod; m++) {
            const u64 q = ctx->mod[m];
            const bool fp = q < (1ULL << 50);
            fpq[m].q = fp ? (double)q : 0.0;
            fpq[m].qinv = fp ? 1.0 / (double)q : 0.0;
            fpq[m].rinv = fpq[m].rinvq = 0.0;
            if (!fp) continue;
            {
                const u64 r = (u64)((((u128)1) << 64) % q), rinv = h_invmod(r, q);
                fpq[m].rinv = (double)rinv, fpq[m].rinvq = (double)rinv / (double)q;
            }
            for (int i = 0; i < n; i++) {
                size_t o = (size_t)m * n + i;
                twd[o] = (double)tw[o], twqd[o] = (double)tw[o] / (double)q;
                itwd[o] = (double)itw[o], itwqd[o] = (double)itw[o] / (double)q;
            }
            nd[m] = (double)ninv[m], nqd[m] = (double)ninv[m] / (double)q;
        }
        ctx->d_fpq = upload(fpq);
        ctx->d_twd = upload(twd), ctx->d_twqd = upload(twqd);
        ctx->d_itwd = upload(itwd), ctx->d_itwqd = upload(itwqd);
        ctx->d_ninvd = upload(nd), ctx->d_ninvqd = upload(nqd);
    }
    std::vector<int> iota(2 * CM_MAX_LIMBS);
    for (int i = 0; i < 2 * CM_MAX_LIMBS; i++) iota[i] = i;
    ctx->d_idx = upload(iota);
    ctx->d_idx_stage = upload(std::vector<int>(CM_NTT_MAX_LIMBS, 0));
    memcpy(ctx->cdt, kGaussCdt, sizeof(kGaussCdt));
    std::vector<u64> cdt(kGaussCdt, kGaussCdt + CM_GAUSS_K);
    ctx->d_cdt = upload(cdt);

    // scratch arena: one key switch at the top level plus operation temporaries
    const int ext = ctx->L + 1 + ctx->K;
    const int beta = (ctx->L + ctx->alpha) / ctx->alpha;
    size_t limbs = (size_t)(ctx->L + 1) + (size_t)beta * ext + 2 * (size_t)ext + 2 * (size_t)(ctx->L + 1) +
                   9 * (size_t)(ctx->L + 1) + 4 +
                   (size_t)CM_KS_BATCH * 2 * (2 * ext + ctx->L + 1);  // batched ModDown of hoisted rotations
    ctx->arena_words = limbs * n;
    if (hipMalloc((void **)&ctx->arena, ctx->arena_words * sizeof(u64)) != hipSuccess) ctx->arena = nullptr;
    if (!ctx->d_modc || !ctx->d_pmont || !ctx->d_ubound || !ctx->d_tw || !ctx->d_twp || !ctx->d_itw || !ctx->d_itwp || !ctx->d_ninv ||
        !ctx->d_ninvp || !ctx->d_idx || !ctx->d_cdt || !ctx->arena) {
        cm_ctx_destroy(ctx);
        return CM_E_NOMEM;
    }
    // encode tables
    ctx->slot_pos.resize(n / 2);
    u64 g = 1;
    for (int j = 0; j < n / 2; j++) {
        ctx->slot_pos[j] = (int)((g - 1) / 2);
        g = g * 5 % (2 * (u64)n);
    }
    ctx->tw_re.resize(n);
    ctx->tw_im.resize(n);
    for (int k = 0; k < n; k++) {
        long double a = M_PIl * k / n;
        ctx->tw_re[k] = (double)cosl(a);
        ctx->tw_im[k] = (double)sinl(a);
    }
    } catch (...) {                  // a failed table upload or host allocation: release what exists
        cm_ctx_destroy(ctx);
        return CM_E_NOMEM;
    }
    cm_ops_device_init();            // per-device addresses of file-scope device arrays, looked up with this device current
    *out = ctx;
    return CM_OK;
}

extern "C" void cm_ctx_destroy(cm_ctx *ctx) {
    if (!ctx) return;
    cm_ops_forget_ctx(ctx);
    for (hipEvent_t e : ctx->prof.pool) hipEventDestroy(e);
    hipFree(ctx->d_modc);
    hipFree(ctx->d_pmont);
    hipFree(ctx->d_ubound);
    hipFree(ctx->d_tw);
    hipFree(ctx->d_twp);
    hipFree(ctx->d_itw);
    hipFree(ctx->d_itwp);
    hipFree(ctx->d_ninv);
    hipFree(ctx->d_ninvp);
    hipFree(ctx->d_fpq), hipFree(ctx->d_twd), hipFree(ctx->d_twqd), hipFree(ctx->d_itwd), hipFree(ctx->d_itwqd);
    hipFree(ctx->d_ninvd), hipFree(ctx->d_ninvqd);
    hipFree(ctx->d_idx);
    hipFree(ctx->d_idx_stage);
    hipFree(ctx->d_cdt);
    hipFree(ctx->arena);
    for (auto &kv : ctx->modup)
        for (auto &t : kv.second) free_conv(t);
    for (auto &kv : ctx->moddown) free_conv(kv.second);
    for (auto &kv : ctx->pinv) hipFree(kv.second);
    for (auto &kv : ctx->qlinv) hipFree(kv.second);
    delete ctx;
}

extern "C" cm_status cm_ctx_moduli(const cm_ctx *ctx, uint64_t *out) {
    if (!ctx || !out) return CM_E_INVAL;
    for (int i = 0; i < ctx->nmod; i++) out[i] = ctx->mod[i];
    return CM_OK;
}
extern "C" size_t cm_ct_words(const cm_ctx *ctx, int32_t level, int32_t ncomp) {
    if (!ctx || level < 0 || level > ctx->L || ncomp < 1) return 0;
    return (size_t)ncomp * (level + 1) * ctx->n;
}
extern "C" size_t cm_pt_words(const cm_ctx *ctx, int32_t level) { return cm_ct_words(ctx, level, 1); }
extern "C" cm_status cm_ctx_gauss_table(const cm_ctx *ctx, uint64_t *out) {
    if (!ctx || !out) return CM_E_INVAL;
    memcpy(out, ctx->cdt, sizeof(ctx->cdt));
    return CM_OK;
}

// ---- canonical embedding (host, double precision) ----------------------------------------------
// In-place radix-2 FFT of length n.  sign = -1: X_k = sum_u x_u exp(-2 pi i u k / n); sign = +1 the
// conjugate kernel.  Roots come from the table omega^k = exp(i pi k / n): exp(2 pi i j / len) = omega^(2 j n / len).
static void fft(const cm_ctx *ctx, std::vector<std::complex<double>> &a, int sign) {
    const size_t n = a.size();
    for (size_t i = 1, j = 0; i < n; i++) {
        size_t bit = n >> 1;
        for (; j & bit; bit >>= 1) j ^= bit;
        j ^= bit;
        if (i < j) std::swap(a[i], a[j]);
    }
    for (size_t len = 2; len <= n; len <<= 1) {
        const size_t stride = 2 * n / len;
        for (size_t s = 0; s < n; s += len)
            for (size_t j = 0; j < len / 2; j++) {
                std::complex<double> w(ctx->tw_re[j * stride], sign * ctx->tw_im[j * stride]);
                std::complex<double> u = a[s + j], v = a[s + j + len / 2] * w;
                a[s + j] = u + v;
                a[s + j + len / 2] = u - v;
            }
    }
}

extern "C" cm_status cm_encode_coeffs(const cm_ctx *ctx, const double *re, const double *im,
                                      size_t nslots, double scale, int64_t *out) {
    if (!ctx || !re || !out || nslots > (size_t)ctx->n / 2 || !(scale > 0)) return CM_E_INVAL;
    CM_TRY
    const int n = ctx->n;
    // values at all primitive 2n-th roots: omega^(2u+1) for slot j at u = slot_pos[j], and the
    // conjugate value at the conjugate root u' = n-1-u; then m_k = Re(FFT(v)_k omega^-k)/n.
    std::vector<std::complex<double>> v(n, 0.0);
    for (size_t j = 0; j < nslots; j++) {
        std::complex<double> z(re[j], im ? im[j] : 0.0);
        v[ctx->slot_pos[j]] = z;
        v[n - 1 - ctx->slot_pos[j]] = std::conj(z);
    }
    fft(ctx, v, -1);
    for (int k = 0; k < n; k++) {
        double m = (v[k].real() * ctx->tw_re[k] + v[k].imag() * ctx->tw_im[k]) / n;
        double x = nearbyint(m * scale);
        if (!(fabs(x) < 9.2e18)) return CM_E_SCALE;
        out[k] = (int64_t)x;
    }
    return CM_OK;
    CM_CATCH
}

// Slot values from centred real coefficients (already divided by the scale).
void decode_host(const cm_ctx *ctx, const std::vector<double> &m, double *re, double *im, size_t nslots) {
    const int n = ctx->n;
    std::vector<std::complex<double>> v(n);
    for (int k = 0; k < n; k++) v[k] = std::complex<double>(m[k] * ctx->tw_re[k], m[k] * ctx->tw_im[k]);
    fft(ctx, v, +1);                 // m(omega^(2u+1)) = sum_k m_k omega^k exp(+2 pi i u k / n)
    for (size_t j = 0; j < nslots; j++) {
        re[j] = v[ctx->slot_pos[j]].real();
        if (im) im[j] = v[ctx->slot_pos[j]].imag();
    }
}
