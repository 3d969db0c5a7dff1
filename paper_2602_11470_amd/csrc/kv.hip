// Encrypted KV cache (Sec. 5): layouts, append, query-times-K and scores-times-V.
//
// Slot (e, h, tau) := (e*H + h)*t + tau with t = S/(H*E): head-interleaved blocks of t slots
// (Sec. 5.3).  The vector of the current token has element [h, e] at (e, h, tau).
//   K ciphertext c   : token c*t + tau at residue tau                                   (Sec. 5.1)
//   score ciphertext : token c*t + tau of head h at (c, h, tau); room for E*t = S/H tokens
//   V ciphertext k   : V[((e + k) mod E)*t + r, h, e] at (e, h, r), stored rotated right by the
//                      giant step of its baby-step/giant-step group                     (Sec. 5.2)
// Every mask is a slot rotation of one of three base masks, so it is obtained from the encoded
// base by the Galois permutation (exact on the integer coefficients).  A mask is encoded at the
// scale of the prime the following rescale removes, so masking leaves the scale unchanged.
#include <math.h>

#include <utility>

#include "kernels.h"

struct cm_kv {
    cm_ctx *ctx = nullptr;
    int S, H, E, t, r_i, r_o, level, max_tokens, ntok, nk_max;
    double scale;
    bool scale_set = false;
    u64 *d_k = nullptr, *d_v = nullptr;     // nk_max / E ciphertexts [2][level+1][n]
    u64 *d_mask_qk = nullptr;               // base: slots (0, h, tau) all h, tau; level-1; multiplier form
    u64 *d_mask_k = nullptr;                // base: slots with residue 0;         level+1
    u64 *d_mask_v = nullptr;                // base: slots (0, h, 0) all h;        level+1
    u64 *d_mask_kg = nullptr;               // every slot;                         level+1  (token-group append)
    u64 *d_mask_vg = nullptr;               // base: slots (0, h, tau) all h, tau; level+1  (token-group append)
    u64 *d_work = nullptr;
    size_t work_words = 0;
    // query-times-K runs CM_KS_BATCH key ciphertexts at a time: tables for raising the third
    // component of their tensor products (level) and the second of their rotated sums (level-1)
    KsManyTables relin_tabs, rot_tabs;
    // sum over the head dims of query-times-K in the extended basis: the ladder cut into runs, every run the hoisted
    // rotations by its subset sums
    bool unrolled = false;
    std::vector<std::vector<long long>> dim_groups;
    // scores-times-V in the same form: giant steps unrolled (one key per multiple of the giant step), the ladder over
    // the residues in runs; tables for raising the second components of up to CM_KS_BATCH inner sums at once
    std::vector<std::vector<long long>> res_groups;
    KsManyTables giant_tabs;
    // query-times-K with the copy mask applied before the last `shared` terms of the sum over the dims: the sums of
    // the key ciphertexts (d_T), their masked combinations A_k (d_A) and the E slot rotations of the mask (d_M)
    // d_Mhat: the transform of d_M along the copy index (the masked sums as a cyclic correlation), with its twiddles
    // the key index: E ciphertexts like d_v, copy b of ciphertext g r_i + j = dim (b + j) of key group b - g r_i;
    // query-times-K from it is the scores-times-V schedule with the query in the place of the scores.  Ciphertext
    // g r_i + j is stored at place j r_o + g: the r_o ciphertexts an append makes from ONE rotation of the new key are
    // then neighbours (one launch reads that rotation once)
    bool indexed = false;
    u64 *d_x = nullptr;
    int shared = 1;
    u64 *d_T = nullptr, *d_A = nullptr, *d_M = nullptr, *d_Mhat = nullptr, *d_tw = nullptr, *d_einv = nullptr;
};

// ceil(L/3) runs of as equal length as possible, the longer ones first; a run lists its non-empty subset sums
static std::vector<std::vector<long long>> ladder_groups(const std::vector<long long> &steps) {
    std::vector<std::vector<long long>> out;
    const size_t L = steps.size(), runs = (L + 2) / 3;
    size_t i = 0;
    for (size_t r = 0; r < runs; r++) {
        const size_t g = L / runs + (r < L % runs ? 1 : 0);
        std::vector<long long> amounts;
        for (unsigned b = 1; b < (1u << g); b++) {
            long long a = 0;
            for (size_t l = 0; l < g; l++)
                if ((b >> l) & 1) a += steps[i + l];
            amounts.push_back(a);
        }
        i += g;
        out.push_back(amounts);
    }
    return out;
}

static int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
}
static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

static cm_status encode_mask(cm_kv *kv, int kind, u64 *dst, int level, const int64_t *coeffs_or_null) {
    cm_ctx *ctx = kv->ctx;
    cm_pt pt;
    pt.dev = dst, pt.mont = 1;
    const double scale = (double)ctx->mod[level];
    if (coeffs_or_null) return cm_pt_from_coeffs(ctx, coeffs_or_null, level, scale, &pt);
    std::vector<double> m(kv->S, 0.0);
    if (kind == 0 || kind == 4)
        for (int i = 0; i < kv->H * kv->t; i++) m[i] = 1.0;
    else if (kind == 1)
        for (int i = 0; i < kv->S; i += kv->t) m[i] = 1.0;
    else if (kind == 3)
        m.assign(kv->S, 1.0);
    else
        for (int h = 0; h < kv->H; h++) m[h * kv->t] = 1.0;
    return cm_encode(ctx, m.data(), nullptr, m.size(), level, scale, &pt);
}

extern "C" cm_status cm_kv_create(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t r_i, int32_t level, double scale,
                                  int32_t max_tokens, cm_kv **out) {
    return cm_kv_create_ex(ctx, heads, dim, r_i, level, scale, max_tokens, 0, out);
}
extern "C" cm_status cm_kv_create_ex(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t r_i, int32_t level, double scale,
                                     int32_t max_tokens, uint32_t flags, cm_kv **out) {
    if (!ctx || !out || heads < 1 || dim < 1 || max_tokens < 1 || (flags & ~(uint32_t)(CM_KV_UNROLLED_LADDERS | CM_KV_KEY_INDEX))) return CM_E_INVAL;
    if (level < 2 || level > ctx->L) return CM_E_LEVEL;
    const int S = ctx->n / 2;
    heads = 1 << ilog2(heads);            // a head count that is not a power of two is padded to the next one
    if (!pow2(dim) || heads * dim > S) return CM_E_LAYOUT;
    cm_kv *kv = new (std::nothrow) cm_kv();
    if (!kv) return CM_E_NOMEM;
    try {
    kv->ctx = ctx, kv->S = S, kv->H = heads, kv->E = dim, kv->t = S / (heads * dim);
    if (r_i == 0) r_i = dim;
    if (!pow2(r_i) || dim % r_i || max_tokens > dim * kv->t) { delete kv; return CM_E_LAYOUT; }
    kv->r_i = r_i, kv->r_o = dim / r_i, kv->level = level, kv->max_tokens = max_tokens, kv->ntok = 0;
    kv->scale = scale > 0 ? scale : ctx->prm.scale;
    kv->nk_max = (max_tokens + kv->t - 1) / kv->t;
    kv->unrolled = (flags & CM_KV_UNROLLED_LADDERS) != 0;
    kv->indexed = (flags & CM_KV_KEY_INDEX) != 0;
    if (kv->unrolled) {
        std::vector<long long> ladder;
        for (int i = 0; i < ilog2(dim); i++) ladder.push_back((long long)(1 << i) * heads * kv->t);
        kv->dim_groups = ladder_groups(ladder);
        std::vector<long long> res;
        for (int l = 0; l < ilog2(kv->t); l++) res.push_back(1LL << l);
        kv->res_groups = ladder_groups(res);
    }
    const size_t n = ctx->n, ctw = 2 * (size_t)(level + 1) * n;
    // work: r_i babies + r_o inner + tensor (1.5 ct) + 5 temporaries, all sized for level+1 inputs of append;
    // or the batch buffers of query-times-K (see kv_qk), whichever is larger
    const size_t ctw_up = 2 * (size_t)(level + 2) * n;
    kv->work_words = (size_t)(kv->r_i + kv->r_o + 8) * ctw_up;
    {
        const KsLevel &kl = ks_level(ctx, level);
        const size_t ln = (size_t)(level + 1) * n, B = CM_KS_BATCH;
        const size_t qk = 5 * ctw + B * (3 * ln + 3 * ctw + ln + (size_t)kl.beta * kl.ext * n + 2 * n + 2 * (size_t)level * n);
        // unrolled: two more sets of CM_KS_BATCH sums in the extended basis of level-1
        const size_t qku = qk + (kv->unrolled ? 2 * B * 2 * (size_t)(level + ctx->K) * n : 0);
        if (qku > kv->work_words) kv->work_words = qku;
        // scores-times-V: babies, inner sums, CM_KS_BATCH tensor sums, two temporaries, the batch's raise buffers
        const size_t sv = (size_t)(kv->r_i + kv->r_o + 2) * ctw + B * (3 * ln + ln + (size_t)kl.beta * kl.ext * n) +
                          (kv->unrolled ? 2 * 2 * (size_t)kl.ext * n : 0);
        if (sv > kv->work_words) kv->work_words = sv;
        // append: mask, one product and its rescale, r_o - 1 shifted inputs, then the batch buffers
        const size_t ap = (size_t)(level + 2) * n + (size_t)(2 + (kv->indexed && kv->r_i > kv->r_o ? kv->r_i : kv->r_o)) * ctw_up +
                          B * (ctw_up + ctw + 2 * n + 2 * (size_t)(level + 1) * n);
        if (ap > kv->work_words) kv->work_words = ap;
    }
    bool ok = hipMalloc((void **)&kv->d_k, (size_t)kv->nk_max * ctw * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_v, (size_t)kv->E * ctw * 8) == hipSuccess &&
              (!kv->indexed || hipMalloc((void **)&kv->d_x, (size_t)kv->E * ctw * 8) == hipSuccess) &&
              hipMalloc((void **)&kv->d_mask_qk, (size_t)level * n * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_mask_k, (size_t)(level + 2) * n * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_mask_v, (size_t)(level + 2) * n * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_mask_kg, (size_t)(level + 2) * n * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_mask_vg, (size_t)(level + 2) * n * 8) == hipSuccess &&
              hipMalloc((void **)&kv->d_work, kv->work_words * 8) == hipSuccess;
    if (ok) ok = ks_many_tables_create(ctx, level, CM_KS_BATCH, &kv->relin_tabs, 3, 2) == CM_OK &&
                 ks_many_tables_create(ctx, level - 1, CM_KS_BATCH, &kv->rot_tabs, 2, 1) == CM_OK &&
                 (!kv->unrolled || ks_many_tables_create(ctx, level, CM_KS_BATCH, &kv->giant_tabs, 2, 1) == CM_OK);
    if (!ok) { cm_kv_destroy(kv); return CM_E_NOMEM; }
    hipMemset(kv->d_k, 0, (size_t)kv->nk_max * ctw * 8);      // an all-zero ciphertext encrypts 0
    hipMemset(kv->d_v, 0, (size_t)kv->E * ctw * 8);
    if (kv->indexed) hipMemset(kv->d_x, 0, (size_t)kv->E * ctw * 8);
    cm_status s = encode_mask(kv, 0, kv->d_mask_qk, level - 1, nullptr);
    if (s == CM_OK && level + 1 <= ctx->L) {
        s = encode_mask(kv, 1, kv->d_mask_k, level + 1, nullptr);
        if (s == CM_OK) s = encode_mask(kv, 2, kv->d_mask_v, level + 1, nullptr);
        if (s == CM_OK) s = encode_mask(kv, 3, kv->d_mask_kg, level + 1, nullptr);
        if (s == CM_OK) s = encode_mask(kv, 4, kv->d_mask_vg, level + 1, nullptr);
    }
    if (s != CM_OK) { cm_kv_destroy(kv); return s; }
    *out = kv;
    return CM_OK;
    } catch (...) {
        cm_kv_destroy(kv);
        return CM_E_NOMEM;
    }
}
extern "C" void cm_kv_destroy(cm_kv *kv) {
    if (!kv) return;
    hipFree(kv->d_k), hipFree(kv->d_v), hipFree(kv->d_x), hipFree(kv->d_mask_qk), hipFree(kv->d_mask_k), hipFree(kv->d_mask_v);
    hipFree(kv->d_mask_kg), hipFree(kv->d_mask_vg);
    hipFree(kv->d_T), hipFree(kv->d_A), hipFree(kv->d_M), hipFree(kv->d_Mhat), hipFree(kv->d_tw), hipFree(kv->d_einv);
    hipFree(kv->d_work);
    ks_many_tables_destroy(&kv->relin_tabs);
    ks_many_tables_destroy(&kv->rot_tabs);
    ks_many_tables_destroy(&kv->giant_tabs);
    delete kv;
}
static u64 rot_g(const cm_kv *kv, long long step);
// d_M[b] = the copy mask of copy b: the base mask rotated right by b copies (a Galois permutation of its rows)
static cm_status build_mask_rows(cm_kv *kv) {
    cm_ctx *ctx = kv->ctx;
    const size_t row = (size_t)kv->level * ctx->n;
    for (int b = 0; b < kv->E; b++) {
        if (b == 0) HIPCHK(hipMemcpy(kv->d_M, kv->d_mask_qk, row * 8, hipMemcpyDeviceToDevice));
        else launch_automorphism(ctx, kv->d_M + b * row, kv->d_mask_qk, kv->level, rot_g(kv, -(long long)b * kv->H * kv->t), 0);
    }
    if (kv->d_Mhat) {
        const int E = kv->E, lv = kv->level;
        std::vector<u64> tw((size_t)lv * 2 * E), einv(lv);
        for (int l = 0; l < lv; l++) {
            const u64 q = ctx->mod[l], w = h_powmod(ctx->psi[l], (u64)(2 * ctx->n / E), q), wi = h_invmod(w, q);
            u64 a = 1, b = 1;
            for (int e = 0; e < E / 2; e++) {
                u64 *f = &tw[((size_t)l * 2 + 0) * E + 2 * e], *g = &tw[((size_t)l * 2 + 1) * E + 2 * e];
                f[0] = a, f[1] = h_shoup(a, q), g[0] = b, g[1] = h_shoup(b, q);
                a = h_mulmod(a, w, q), b = h_mulmod(b, wi, q);
            }
            einv[l] = h_mulmod(h_invmod((u64)E % q, q), (u64)(((u128)1 << 64) % q), q);
        }
        HIPCHK(hipMemcpy(kv->d_tw, tw.data(), tw.size() * 8, hipMemcpyHostToDevice));
        HIPCHK(hipMemcpy(kv->d_einv, einv.data(), einv.size() * 8, hipMemcpyHostToDevice));
        launch_mask_ntt_setup(ctx, kv->d_Mhat, kv->d_M, kv->d_tw, kv->d_einv, E, lv, 0);
    }
    HIPCHK(hipDeviceSynchronize());
    return CM_OK;
}
// Parity hook: replace a base mask by given integer coefficients (kind 0: query-times-K mask at
// level-1; 1: residue mask at level+1; 2: value mask at level+1; 3 and 4: the all-ones and value
// masks of the token-group append at level+1), host coeffs[n].
extern "C" cm_status cm_kv_set_mask(cm_kv *kv, int32_t kind, const int64_t *coeffs) {
    if (!kv || !coeffs || kind < 0 || kind > 4) return CM_E_INVAL;
    if (kind > 0 && kv->level + 1 > kv->ctx->L) return CM_E_LEVEL;
    CM_TRY
    u64 *dst = kind == 0 ? kv->d_mask_qk : kind == 1 ? kv->d_mask_k : kind == 2 ? kv->d_mask_v
             : kind == 3 ? kv->d_mask_kg : kv->d_mask_vg;
    CMCHK(encode_mask(kv, kind, dst, kind == 0 ? kv->level - 1 : kv->level + 1, coeffs));
    return kind == 0 && kv->d_M ? build_mask_rows(kv) : CM_OK;
    CM_CATCH
}
// How many terms of the sum over the dims of query-times-K are taken AFTER the copy mask, by rotations shared by all
// key ciphertexts (1 = none).  Rebuilds the runs of the per-ciphertext part and allocates the buffers of the shared part.
extern "C" cm_status cm_kv_set_shared_dims(cm_kv *kv, int32_t shared) {
    if (!kv || !kv->unrolled) return CM_E_INVAL;
    if (!pow2(shared) || shared > kv->E) return CM_E_LAYOUT;
    CM_TRY
    cm_ctx *ctx = kv->ctx;
    std::vector<long long> ladder;
    for (int i = 0; i < ilog2(kv->E / shared); i++) ladder.push_back((long long)(shared << i) * kv->H * kv->t);
    auto release = [&]() {
        hipFree(kv->d_T), hipFree(kv->d_A), hipFree(kv->d_M), hipFree(kv->d_Mhat), hipFree(kv->d_tw), hipFree(kv->d_einv);
        kv->d_T = kv->d_A = kv->d_M = kv->d_Mhat = kv->d_tw = kv->d_einv = nullptr;
    };
    release();
    kv->shared = 1;
    if (shared > 1) {
        const size_t n = ctx->n, ctw1 = 2 * (size_t)kv->level * n;
        const bool ntt = mask_ntt_supported(kv->E);
        if (hipMalloc((void **)&kv->d_T, (size_t)kv->nk_max * ctw1 * 8) != hipSuccess ||
            hipMalloc((void **)&kv->d_A, (size_t)shared * ctw1 * 8) != hipSuccess ||
            hipMalloc((void **)&kv->d_M, (size_t)kv->E * kv->level * n * 8) != hipSuccess ||
            (ntt && (hipMalloc((void **)&kv->d_Mhat, (size_t)kv->E * kv->level * n * 8) != hipSuccess ||
                     hipMalloc((void **)&kv->d_tw, (size_t)kv->level * 2 * kv->E * 8) != hipSuccess ||
                     hipMalloc((void **)&kv->d_einv, (size_t)kv->level * 8) != hipSuccess))) {
            release();
            std::vector<long long> full;
            for (int i = 0; i < ilog2(kv->E); i++) full.push_back((long long)(1 << i) * kv->H * kv->t);
            kv->dim_groups = ladder_groups(full);
            return CM_E_NOMEM;
        }
    }
    kv->shared = shared;
    kv->dim_groups = ladder_groups(ladder);
    return shared > 1 ? build_mask_rows(kv) : CM_OK;
    CM_CATCH
}

static std::vector<int> kv_all_steps(const cm_kv *kv) {
    std::vector<int> s;
    for (int i = 0; i < ilog2(kv->t); i++) s.push_back(-(1 << i));                         // replicate q
    if (kv->indexed) {
        // query-times-K runs on the index: baby and giant steps below, no sum over the dims
    } else if (kv->unrolled) {
        for (const auto &grp : kv->dim_groups)
            for (long long a : grp) s.push_back((int)a);                                       // sum over dims, run by run
        for (int k = 1; k < kv->shared; k++) s.push_back(k * kv->H * kv->t);                   // ... and its shared part
    } else {
        for (int i = 0; i < ilog2(kv->E); i++) s.push_back((1 << i) * kv->H * kv->t);      // sum over dims
    }
    for (int j = 1; j < kv->r_i; j++) s.push_back(j * kv->H * kv->t);                      // score baby steps
    if (kv->unrolled) {
        for (int g = 1; g < kv->r_o; g++) s.push_back(g * kv->r_i * kv->H * kv->t);        // every multiple of the giant step
        for (const auto &grp : kv->res_groups)
            for (long long a : grp) s.push_back((int)a);                                       // reduce residues, run by run
    } else {
        if (kv->r_o > 1) s.push_back(kv->r_i * kv->H * kv->t);                             // score giant step
        for (int l = 0; l < ilog2(kv->t); l++) s.push_back(1 << l);                        // reduce residues
    }
    for (int g = 1; g < kv->r_o; g++) s.push_back(-(g * kv->r_i * kv->H * kv->t));         // append shifts
    return s;
}
extern "C" int32_t cm_kv_steps(const cm_kv *kv, int32_t *steps, int32_t cap) {
    if (!kv) return 0;
    try {
        auto s = kv_all_steps(kv);
        for (int i = 0; i < (int)s.size() && i < cap && steps; i++) steps[i] = s[i];
        return (int32_t)s.size();
    } catch (...) {
        return 0;
    }
}
extern "C" int32_t cm_kv_tokens(const cm_kv *kv) { return kv ? kv->ntok : -1; }
extern "C" cm_status cm_kv_set_tokens(cm_kv *kv, int32_t ntok) {
    if (!kv || ntok < 0 || ntok > kv->max_tokens) return CM_E_INVAL;
    kv->ntok = ntok;
    return CM_OK;
}

static size_t kv_ctw(const cm_kv *kv) { return 2 * (size_t)(kv->level + 1) * kv->ctx->n; }
static int x_place(const cm_kv *kv, int k) { return (k % kv->r_i) * kv->r_o + k / kv->r_i; }

extern "C" cm_status cm_kv_load(cm_ctx *ctx, cm_kv *kv, int32_t which, int32_t idx, const cm_ct *ct, void *stream) {
    if (!ctx || !kv || kv->ctx != ctx || !ct || !ct->dev || ct->ncomp != 2) return CM_E_INVAL;
    if (ct->level != kv->level) return CM_E_LEVEL;
    if (kv->scale_set && fabs(ct->scale / kv->scale - 1) > 1e-9) return CM_E_SCALE;
    if (which != CM_QK && which != CM_SV && !(which == CM_KV_INDEX && kv->indexed)) return CM_E_INVAL;
    if (idx < 0 || idx >= (which == CM_QK ? kv->nk_max : kv->E)) return CM_E_LAYOUT;
    u64 *dst = (which == CM_QK ? kv->d_k : which == CM_SV ? kv->d_v : kv->d_x) + (size_t)(which == CM_KV_INDEX ? x_place(kv, idx) : idx) * kv_ctw(kv);
    HIPCHK(hipMemcpyAsync(dst, ct->dev, kv_ctw(kv) * 8, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    kv->scale = ct->scale, kv->scale_set = true;
    return CM_OK;
}
extern "C" cm_status cm_kv_export(cm_ctx *ctx, const cm_kv *kv, int32_t which, int32_t idx, uint64_t *out) {
    if (!ctx || !kv || !out) return CM_E_INVAL;
    if (which != CM_QK && which != CM_SV && !(which == CM_KV_INDEX && kv->indexed)) return CM_E_INVAL;
    if (idx < 0 || idx >= (which == CM_QK ? kv->nk_max : kv->E)) return CM_E_LAYOUT;
    cm_ct ct;
    ct.dev = (which == CM_QK ? kv->d_k : which == CM_SV ? kv->d_v : kv->d_x) + (size_t)(which == CM_KV_INDEX ? x_place(kv, idx) : idx) * kv_ctw(kv);
    ct.level = kv->level, ct.ncomp = 2, ct.scale = kv->scale;
    return cm_ct_export(ctx, &ct, out);
}

static u64 rot_g(const cm_kv *kv, long long step) {
    long long S = kv->S;
    return galois_of_step(kv->ctx, (int)(((step % S) + S) % S));
}

// One token (k_new / v_new hold it at residue ntok mod t), or, group = true, the t tokens of the
// next K ciphertext at once (Sec. 5.4: token c*t + tau at residue tau, which is already the layout
// of K ciphertext c; the V masks take whole block rows, all residues together).
static cm_status kv_append(cm_ctx *ctx, const cm_evk *evk, cm_kv *kv, const cm_ct *k_new, const cm_ct *v_new,
                           bool group, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !kv || kv->ctx != ctx || !k_new || !v_new || !k_new->dev || !v_new->dev || !evk_fits(ctx, evk)) return CM_E_INVAL;
    if (k_new->ncomp != 2 || v_new->ncomp != 2) return CM_E_INVAL;
    CM_TRY
    const int lv = kv->level + 1;
    if (lv > ctx->L || k_new->level != lv || v_new->level != lv) return CM_E_LEVEL;
    if (kv->ntok >= kv->max_tokens) return CM_E_LAYOUT;
    if (group && (kv->ntok % kv->t || kv->ntok + kv->t > kv->max_tokens)) return CM_E_LAYOUT;
    if (kv->scale_set && (fabs(k_new->scale / kv->scale - 1) > 1e-9 || fabs(v_new->scale / kv->scale - 1) > 1e-9))
        return CM_E_SCALE;
    if (fabs(k_new->scale / v_new->scale - 1) > 1e-9) return CM_E_SCALE;
    for (int g = 1; g < kv->r_o; g++)
        if (!find_key(evk, rot_g(kv, -(long long)g * kv->r_i * kv->H * kv->t))) return CM_E_NOKEY;
    for (int j = 1; j < kv->r_i && kv->indexed; j++)
        if (!find_key(evk, rot_g(kv, (long long)j * kv->H * kv->t))) return CM_E_NOKEY;
    hipStream_t st = (hipStream_t)stream;
    const size_t n = ctx->n, ctw_up = 2 * (size_t)(lv + 1) * n, ctw = kv_ctw(kv);
    const int tok = kv->ntok, c = tok / kv->t, tau = tok % kv->t;
    u64 *mask = kv->d_work, *prod = mask + (size_t)(lv + 1) * n, *res = prod + ctw_up, *shifted = res + ctw_up;
    // K: K_c += rescale(k_new * mask_tau), mask_tau = residue-0 mask rotated right by tau (a group: all ones)
    if (!group) launch_automorphism(ctx, mask, kv->d_mask_k, lv + 1, rot_g(kv, -tau), st);
    launch_mul_pt(ctx, prod, k_new->dev, group ? kv->d_mask_kg : mask, 2, lv + 1, st);
    CMCHK(rescale_into(ctx, prod, 2, lv, kv->d_k + (size_t)c * ctw, st, nullptr, nullptr, true));
    // V: the new vector shifted right by each giant step, then one masked product per V ciphertext
    if (kv->r_o > 1) {                                       // rotations of one ciphertext: one raise for all of them
        u64 *digits = arena_digits(ctx);
        CMCHK(ks_raise(ctx, v_new->dev + (size_t)(lv + 1) * n, lv, digits, st));
        std::vector<const u64 *> keys;
        std::vector<u64> gs;
        std::vector<u64 *> dst;
        for (int g = 1; g < kv->r_o; g++) {
            const u64 gal = rot_g(kv, -(long long)g * kv->r_i * kv->H * kv->t);
            keys.push_back(find_key(evk, gal)), gs.push_back(gal), dst.push_back(shifted + (size_t)(g - 1) * ctw_up);
        }
        CMCHK(ks_apply_many(ctx, digits, lv, kv->r_o - 1, keys.data(), gs.data(), v_new->dev, dst.data(), st));
    }
    // CM_KS_BATCH value ciphertexts at a time: their masked products in one launch, one stacked rescale,
    // one stacked addition (consecutive value ciphertexts are contiguous)
    u64 *prods = shifted + (size_t)(kv->r_o > 1 ? kv->r_o - 1 : 0) * ctw_up, *ress = prods + (size_t)CM_KS_BATCH * ctw_up;
    u64 *last = ress + (size_t)CM_KS_BATCH * ctw, *red = last + (size_t)CM_KS_BATCH * 2 * n;
    for (int kb = 0; kb < kv->E; kb += CM_KS_BATCH) {
        const int m = kv->E - kb < CM_KS_BATCH ? kv->E - kb : CM_KS_BATCH;
        MulPtBatch mb;
        for (int r = 0; r < m; r++) {
            const int k = kb + r, g = k / kv->r_i;
            long long a = (long long)(((c - k) % kv->E + kv->E) % kv->E) * kv->H * kv->t + tau +
                          (long long)g * kv->r_i * kv->H * kv->t;
            mb.src[r] = g == 0 ? v_new->dev : shifted + (size_t)(g - 1) * ctw_up;
            mb.g[r] = (unsigned)rot_g(kv, -a);
        }
        // consecutive value ciphertexts are contiguous: the rescale adds its result onto them
        const u64 *vmask = group ? kv->d_mask_vg : kv->d_mask_v;
        if (rescale_masked_into(ctx, mb, m, vmask, lv, kv->d_v + (size_t)kb * ctw, st, last, red, true)) continue;
        launch_mul_pt_rot_batch(ctx, prods, mb, m, vmask, lv + 1, st);
        CMCHK(rescale_into(ctx, prods, 2 * m, lv, kv->d_v + (size_t)kb * ctw, st, last, red, true));
    }
    if (kv->indexed) {
        // index: X_{g r_i + j} += rescale(mask * Rot(k_new, j B)), mask = copy (c + g r_i) mod E at residue tau (a group: the
        // whole copy); the baby rotations of the new key are hoisted, the masked products go eight per launch
        if (kv->r_i > 1) {
            u64 *digits = arena_digits(ctx);
            CMCHK(ks_raise(ctx, k_new->dev + (size_t)(lv + 1) * n, lv, digits, st));
            std::vector<const u64 *> keys;
            std::vector<u64> gs;
            std::vector<u64 *> dst;
            for (int j = 1; j < kv->r_i; j++) {
                const u64 gal = rot_g(kv, (long long)j * kv->H * kv->t);
                keys.push_back(find_key(evk, gal)), gs.push_back(gal), dst.push_back(shifted + (size_t)(j - 1) * ctw_up);
            }
            CMCHK(ks_apply_many(ctx, digits, lv, kv->r_i - 1, keys.data(), gs.data(), k_new->dev, dst.data(), st));
        }
        u64 *xp = shifted + (size_t)(kv->r_i > 1 ? kv->r_i - 1 : 0) * ctw_up, *xr = xp + (size_t)CM_KS_BATCH * ctw_up;
        u64 *xl = xr + (size_t)CM_KS_BATCH * ctw, *xd = xl + (size_t)CM_KS_BATCH * 2 * n;
        for (int kb = 0; kb < kv->E; kb += CM_KS_BATCH) {
            const int m = kv->E - kb < CM_KS_BATCH ? kv->E - kb : CM_KS_BATCH;
            MulPtBatch mb;
            for (int r = 0; r < m; r++) {
                const int place = kb + r, j = place / kv->r_o, g = place % kv->r_o;      // index ciphertext g r_i + j
                const long long a = (long long)((c + g * kv->r_i) % kv->E) * kv->H * kv->t + tau;
                mb.src[r] = j == 0 ? k_new->dev : shifted + (size_t)(j - 1) * ctw_up;
                mb.g[r] = (unsigned)rot_g(kv, -a);
            }
            const u64 *xmask = group ? kv->d_mask_vg : kv->d_mask_v;
            if (rescale_masked_into(ctx, mb, m, xmask, lv, kv->d_x + (size_t)kb * ctw, st, xl, xd, true)) continue;
            launch_mul_pt_rot_batch(ctx, xp, mb, m, xmask, lv + 1, st);
            CMCHK(rescale_into(ctx, xp, 2 * m, lv, kv->d_x + (size_t)kb * ctw, st, xl, xd, true));
        }
    }
    kv->ntok += group ? kv->t : 1;
    kv->scale = k_new->scale * (double)ctx->mod[lv] / (double)ctx->mod[lv];
    kv->scale_set = true;
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
extern "C" cm_status cm_kv_append(cm_ctx *ctx, const cm_evk *evk, cm_kv *kv, const cm_ct *k_new, const cm_ct *v_new,
                                  void *stream) {
    return kv_append(ctx, evk, kv, k_new, v_new, false, stream);
}
extern "C" cm_status cm_kv_append_group(cm_ctx *ctx, const cm_evk *evk, cm_kv *kv, const cm_ct *k_grp,
                                        const cm_ct *v_grp, void *stream) {
    return kv_append(ctx, evk, kv, k_grp, v_grp, true, stream);
}

// every key query-times-K needs is there (checked before anything is enqueued)
static cm_status kv_qk_keys(const cm_evk *evk, const cm_kv *kv, bool replicate) {
    if (kv->level < 2) return CM_E_LEVEL;
    if (!find_key(evk, 0)) return CM_E_NOKEY;
    for (int i = 0; i < ilog2(kv->t) && replicate; i++) if (!find_key(evk, rot_g(kv, -(1 << i)))) return CM_E_NOKEY;
    if (kv->unrolled) {
        for (const auto &grp : kv->dim_groups)
            for (long long a : grp) if (!find_key(evk, rot_g(kv, a))) return CM_E_NOKEY;
        for (int k = 1; k < kv->shared; k++) if (!find_key(evk, rot_g(kv, (long long)k * kv->H * kv->t))) return CM_E_NOKEY;
    } else {
        for (int i = 0; i < ilog2(kv->E); i++) if (!find_key(evk, rot_g(kv, (long long)(1 << i) * kv->H * kv->t))) return CM_E_NOKEY;
    }
    return (kv->ntok + kv->t - 1) / kv->t < 1 ? CM_E_LAYOUT : CM_OK;
}
static cm_status kv_qk(cm_ctx *ctx, const cm_evk *evk, const cm_kv *kv, const cm_ct *in, cm_ct *out, hipStream_t st,
                       bool replicate) {
    const int lv = kv->level, limbs = lv + 1;
    CMCHK(kv_qk_keys(evk, kv, replicate));
    const size_t n = ctx->n, ctw = kv_ctw(kv), ln = (size_t)limbs * n;
    const u64 *relin = find_key(evk, 0);
    const int nk = (kv->ntok + kv->t - 1) / kv->t;
    // The key ciphertexts are independent until the final sum, so CM_KS_BATCH of them go through every
    // step together: their raises, their ModDowns and their rescales are single batches of launches.
    const KsLevel &kl = ks_level(ctx, lv), &kl1 = ks_level(ctx, lv - 1);
    const size_t B = CM_KS_BATCH, ln1 = (size_t)lv * n, ctw1 = 2 * ln1;
    u64 *cq = kv->d_work, *tmp = cq + ctw, *acc = tmp + ctw, *mask = acc + ctw;
    u64 *TB = mask + ctw, *PB = TB + B * 3 * ln, *RB0 = PB + B * ctw, *RB1 = RB0 + B * ctw, *ksin = RB1 + B * ctw;
    u64 *digits = ksin + B * ln, *last = digits + B * (size_t)kl.beta * kl.ext * n, *red = last + B * 2 * n;
    u64 *bu = arena_batch_sums(ctx);
    const size_t rw1 = 2 * (size_t)kl1.ext * n;                   // one sum in the extended basis of level-1
    u64 *XA = red + B * 2 * (size_t)lv * n, *XB = XA + B * rw1;   // unrolled form only
    HIPCHK(hipMemcpyAsync(cq, in->dev, ctw * 8, hipMemcpyDeviceToDevice, st));
    for (int i = 0; i < ilog2(kv->t) && replicate; i++) {        // replicate q over the t residues
        u64 g = rot_g(kv, -(1 << i));
        CMCHK(rotate_into(ctx, find_key(evk, g), cq, lv, g, tmp, st, cq));      // tmp = cq + Rot(cq)
        std::swap(cq, tmp);
    }
    for (int c0 = 0; c0 < nk; c0 += CM_KS_BATCH) {
        const int m = nk - c0 < CM_KS_BATCH ? nk - c0 : CM_KS_BATCH;
        const u64 *adds[CM_KS_BATCH], *accs[CM_KS_BATCH];
        u64 *outs[CM_KS_BATCH];
        // tensor products, relinearised together
        launch_tensor_batch(ctx, TB, cq, kv->d_k + (size_t)c0 * ctw, m, limbs, st);
        CMCHK(ks_raise_many(ctx, kv->relin_tabs, TB, ksin, digits, st, m, 0));
        const size_t ublk = 2 * (size_t)kl.ext * n, dblk = (size_t)kl.beta * kl.ext * n;
        IpBatch ip;
        ip.nz = m, ip.nsum = 1;
        for (int r = 0; r < m; r++) {
            ip.it[r].dig = digits + r * dblk, ip.it[r].key = relin, ip.it[r].c0 = nullptr, ip.it[r].g = 0;
            ip.out[r] = bu + r * ublk, ip.extra[r] = nullptr;
            adds[r] = TB + r * 3 * ln, outs[r] = PB + r * ctw;
        }
        launch_inner_product_shared_key(ctx, ip, kl.beta, lv, st);
        CMCHK(moddown_batch_into(ctx, bu, lv, m, adds, 2, 0, nullptr, outs, st));
        // with shared rotations the sums of the key ciphertexts are kept (d_T) until all of them are there
        u64 *r0 = kv->shared > 1 ? kv->d_T + (size_t)c0 * ctw1 : RB0, *r1 = RB1;
        CMCHK(rescale_into(ctx, PB, 2 * m, lv, r0, st, last, red));        // stacked: [m][2][lv+1] -> [m][2][lv]
        const size_t ublk1 = 2 * (size_t)kl1.ext * n, dblk1 = (size_t)kl1.beta * kl1.ext * n;
        if (kv->unrolled && !kv->dim_groups.empty()) {
            // sum over the E dims in the extended basis: R = (P c0, P c1); every run adds the hoisted rotations of R by
            // its subset sums (one raise of ModDown(R1) per run, one launch per rotation amount over all m ciphertexts,
            // the key read once per launch); one ModDown of both components at the end
            launch_raise_by_P(ctx, XA, r0, lv - 1, st, m);
            u64 *cur = XA, *nxt = XB;
            for (size_t gi = 0; gi < kv->dim_groups.size(); gi++) {
                if (gi) {                                       // the first run's second components are the exact c1
                    for (int r = 0; r < m; r++) outs[r] = r0 + r * ctw1;
                    CMCHK(moddown_second_keep_many(ctx, cur, lv - 1, m, outs, st));
                }
                CMCHK(ks_raise_many(ctx, kv->rot_tabs, r0, ksin, digits, st, m, 0));
                bool first = true;
                const auto &grp = kv->dim_groups[gi];
                for (size_t a0 = 0; a0 < grp.size();) {
                    // up to IP_MULTI_KEYS rotation amounts per launch (their keys in registers, the running sum written
                    // once); the remainder, or everything if there are too many digits for that, one amount per launch
                    const int na = (int)(grp.size() - a0 < (size_t)IP_MULTI_KEYS ? grp.size() - a0 : IP_MULTI_KEYS);
                    for (int r = 0; r < m; r++) {
                        ip.it[r].dig = digits + r * dblk1;
                        ip.it[r].c0 = cur + r * rw1, ip.it[r].c0_ext = 1;
                        ip.out[r] = nxt + r * rw1, ip.extra[r] = first ? cur + r * rw1 : nxt + r * rw1;
                    }
                    IpKeys ks;
                    for (int a = 0; a < na; a++) ks.g[a] = (unsigned)rot_g(kv, grp[a0 + a]), ks.key[a] = find_key(evk, ks.g[a]);
                    if (na >= 2 && launch_inner_product_multi_key(ctx, ip, ks, na, kl1.beta, lv - 1, st)) {
                        a0 += na;
                    } else {
                        for (int r = 0; r < m; r++) ip.it[r].key = ks.key[0];
                        launch_inner_product_shared_key(ctx, ip, kl1.beta, lv - 1, st, ks.g[0]);
                        a0 += 1;
                    }
                    first = false;
                }
                std::swap(cur, nxt);
            }
            for (int r = 0; r < m; r++) outs[r] = r0 + r * ctw1, ip.it[r].c0 = nullptr, ip.it[r].c0_ext = 0, ip.extra[r] = nullptr;
            CMCHK(moddown_batch_into(ctx, cur, lv - 1, m, nullptr, 0, 0, nullptr, outs, st));
        }
        for (int i = 0; i < ilog2(kv->E) && !kv->unrolled; i++) {                 // sum over the E dims of every head
            u64 g = rot_g(kv, (long long)(1 << i) * kv->H * kv->t);
            const u64 *key = find_key(evk, g);
            CMCHK(ks_raise_many(ctx, kv->rot_tabs, r0, ksin, digits, st, m, g));
            for (int r = 0; r < m; r++) {
                ip.it[r].dig = digits + r * dblk1, ip.it[r].key = key, ip.out[r] = bu + r * ublk1;
                adds[r] = accs[r] = r0 + r * ctw1, outs[r] = r1 + r * ctw1;
            }
            launch_inner_product_shared_key(ctx, ip, kl1.beta, lv - 1, st);
            CMCHK(moddown_batch_into(ctx, bu, lv - 1, m, adds, 1, g, accs, outs, st));
            std::swap(r0, r1);
        }
        if (kv->shared == 1) {
            // keep copy e = c of every key ciphertext's sums: base mask rotated right by c*H*t; one launch
            MulPtBatch mb;
            for (int r = 0; r < m; r++) mb.src[r] = nullptr, mb.g[r] = (unsigned)rot_g(kv, -(long long)((c0 + r) % kv->E) * kv->H * kv->t);
            launch_mac_pt_rot_batch(ctx, acc, r0, mb, m, kv->d_mask_qk, lv, c0 > 0, st);
        }
    }
    if (kv->shared > 1) {
        // A_k = sum_c mask_{c+k} T_c; scores = ModDown( P A_0 + sum_{k >= 1} RotRaised(A_k, k H t) ): shared - 1 rotations
        // for the whole cache, CM_KS_BATCH of them raised and summed per launch
        // directly (nk * shared products per coefficient) or, when that is more than the transform's E (log2 E + 1) by a
        // wide margin, as a cyclic correlation along the copy index
        if (kv->d_Mhat && (long long)nk * kv->shared >= 16LL * kv->E)
            launch_mask_ntt(ctx, kv->d_A, kv->d_T, kv->d_Mhat, kv->d_tw, kv->d_einv, nk, kv->E, kv->shared, lv, st);
        else
            launch_mask_circulant(ctx, kv->d_A, kv->d_T, kv->d_M, nk, kv->E, kv->shared, lv, st);
        const size_t dblk1 = (size_t)kl1.beta * kl1.ext * n;
        u64 *cur = XA, *nxt = XB;
        launch_raise_by_P(ctx, cur, kv->d_A, lv - 1, st, 1);
        for (int k0 = 1; k0 < kv->shared; k0 += CM_KS_BATCH) {
            const int m = kv->shared - k0 < CM_KS_BATCH ? kv->shared - k0 : CM_KS_BATCH;
            CMCHK(ks_raise_many(ctx, kv->rot_tabs, kv->d_A + (size_t)k0 * ctw1, ksin, digits, st, m, 0));
            IpBatch b;
            b.nz = 1, b.nsum = m;
            for (int r = 0; r < m; r++) {
                const u64 gal = rot_g(kv, (long long)(k0 + r) * kv->H * kv->t);
                b.it[r].dig = digits + r * dblk1, b.it[r].key = find_key(evk, gal), b.it[r].g = (unsigned)gal;
                b.it[r].c0 = kv->d_A + (size_t)(k0 + r) * ctw1, b.it[r].c0_ext = 0;
            }
            b.out[0] = nxt, b.extra[0] = cur;
            launch_inner_product_batch(ctx, b, kl1.beta, lv - 1, st);
            std::swap(cur, nxt);
        }
        CMCHK(moddown_into(ctx, cur, lv - 1, nullptr, 0, 0, acc, nullptr, st));
    }
    CMCHK(rescale_into(ctx, acc, 2, lv - 1, out->dev, st));
    out->level = lv - 2, out->ncomp = 2;
    out->scale = in->scale * kv->scale / (double)ctx->mod[lv];      // the mask scale cancels the second rescale
    RETURN_LAUNCH_STATUS();
}

// array = the value ciphertexts, or the key index with the query in the place of the scores (replicate: the query is
// first copied to all residues, as query-times-K does)
static cm_status kv_sv_keys(const cm_evk *evk, const cm_kv *kv, bool reduce, bool replicate) {
    for (int i = 0; i < ilog2(kv->t) && replicate; i++) if (!find_key(evk, rot_g(kv, -(1 << i)))) return CM_E_NOKEY;
    if (!find_key(evk, 0)) return CM_E_NOKEY;
    const long long Ht = (long long)kv->H * kv->t;
    for (int j = 1; j < kv->r_i; j++) if (!find_key(evk, rot_g(kv, j * Ht))) return CM_E_NOKEY;
    if (kv->unrolled) {
        for (int g = 1; g < kv->r_o; g++) if (!find_key(evk, rot_g(kv, (long long)g * kv->r_i * Ht))) return CM_E_NOKEY;
        for (const auto &grp : kv->res_groups)
            for (long long a : grp) if (reduce && !find_key(evk, rot_g(kv, a))) return CM_E_NOKEY;
    } else {
        if (kv->r_o > 1 && !find_key(evk, rot_g(kv, kv->r_i * Ht))) return CM_E_NOKEY;
        for (int l = 0; l < ilog2(kv->t) && reduce; l++) if (!find_key(evk, rot_g(kv, 1 << l))) return CM_E_NOKEY;
    }
    return CM_OK;
}
static cm_status kv_sv(cm_ctx *ctx, const cm_evk *evk, const cm_kv *kv, const cm_ct *in, cm_ct *out, hipStream_t st,
                       bool reduce, const u64 *array, bool replicate) {
    const int lv = kv->level, limbs = lv + 1;
    CMCHK(kv_sv_keys(evk, kv, reduce, replicate));
    const size_t n = ctx->n, ctw = kv_ctw(kv), ln = (size_t)limbs * n;
    const u64 *relin = find_key(evk, 0);
    const long long Ht = (long long)kv->H * kv->t;
    const KsLevel &kl = ks_level(ctx, lv);
    const size_t B = CM_KS_BATCH, dblk = (size_t)kl.beta * kl.ext * n, ublk = 2 * (size_t)kl.ext * n;
    u64 *babies = kv->d_work, *inner = babies + (size_t)kv->r_i * ctw, *T = inner + (size_t)kv->r_o * ctw,
        *tmp = T + B * 3 * ln, *R = tmp + ctw, *ksin = R + ctw, *bdigits = ksin + B * ln;
    u64 *digits = arena_digits(ctx);
    HIPCHK(hipMemcpyAsync(babies, in->dev, ctw * 8, hipMemcpyDeviceToDevice, st));
    if (replicate) {
        u64 *cq = babies, *alt = tmp;
        for (int i = 0; i < ilog2(kv->t); i++) {
            const u64 g = rot_g(kv, -(1 << i));
            CMCHK(rotate_into(ctx, find_key(evk, g), cq, lv, g, alt, st, cq));      // alt = cq + Rot(cq)
            std::swap(cq, alt);
        }
        if (cq != babies) HIPCHK(hipMemcpyAsync(babies, cq, ctw * 8, hipMemcpyDeviceToDevice, st));
    }
    if (kv->r_i > 1) {
        CMCHK(ks_raise(ctx, babies + ln, lv, digits, st));
        std::vector<const u64 *> keys;
        std::vector<u64> gs;
        std::vector<u64 *> dst;
        for (int j = 1; j < kv->r_i; j++) {
            keys.push_back(find_key(evk, rot_g(kv, j * Ht)));
            gs.push_back(rot_g(kv, j * Ht));
            dst.push_back(babies + (size_t)j * ctw);
        }
        CMCHK(ks_apply_many(ctx, digits, lv, kv->r_i - 1, keys.data(), gs.data(), babies, dst.data(), st));
    }
    // inner_g = relinearise(sum_j baby_j (x) V_{g r_i + j}): the sums of up to CM_KS_BATCH groups by one launch, their
    // third components raised together, one inner-product launch with the relinearisation key read once, one ModDown
    for (int g0 = 0; g0 < kv->r_o; g0 += CM_KS_BATCH) {
        const int m = kv->r_o - g0 < CM_KS_BATCH ? kv->r_o - g0 : CM_KS_BATCH;
        if (array == kv->d_x) launch_tensor_sum(ctx, T, babies, array + (size_t)g0 * ctw, kv->r_i, m, limbs, st, 1, kv->r_o);
        else launch_tensor_sum(ctx, T, babies, array + (size_t)g0 * kv->r_i * ctw, kv->r_i, m, limbs, st);
        CMCHK(ks_raise_many(ctx, kv->relin_tabs, T, ksin, bdigits, st, m, 0));
        u64 *bu = arena_batch_sums(ctx);
        IpBatch ip;
        ip.nz = m, ip.nsum = 1;
        const u64 *adds[CM_KS_BATCH];
        u64 *outs[CM_KS_BATCH];
        for (int r = 0; r < m; r++) {
            ip.it[r].dig = bdigits + r * dblk, ip.it[r].key = relin, ip.it[r].c0 = nullptr, ip.it[r].g = 0;
            ip.out[r] = bu + r * ublk, ip.extra[r] = nullptr;
            adds[r] = T + (size_t)r * 3 * ln, outs[r] = inner + (size_t)(g0 + r) * ctw;
        }
        launch_inner_product_shared_key(ctx, ip, kl.beta, lv, st);
        CMCHK(moddown_batch_into(ctx, bu, lv, m, adds, 2, 0, nullptr, outs, st));
    }
    if (kv->unrolled) {
        // sum_g Rot(inner_g, g G) next to P inner_0, then the ladder over the residues, all in the extended basis;
        // one ModDown, then the rescale
        const size_t rw = 2 * (size_t)kl.ext * n;
        u64 *cur = bdigits + B * dblk, *nxt = cur + rw;
        launch_raise_by_P(ctx, cur, inner, lv, st);
        for (int g0 = 1; g0 < kv->r_o; g0 += CM_KS_BATCH) {
            const int m = kv->r_o - g0 < CM_KS_BATCH ? kv->r_o - g0 : CM_KS_BATCH;
            CMCHK(ks_raise_many(ctx, kv->giant_tabs, inner + (size_t)g0 * ctw, ksin, bdigits, st, m, 0));
            IpBatch b;
            b.nz = 1, b.nsum = m;
            for (int r = 0; r < m; r++) {
                const u64 gal = rot_g(kv, (long long)(g0 + r) * kv->r_i * Ht);
                b.it[r].dig = bdigits + r * dblk, b.it[r].key = find_key(evk, gal), b.it[r].g = (unsigned)gal;
                b.it[r].c0 = inner + (size_t)(g0 + r) * ctw, b.it[r].c0_ext = 0;
            }
            b.out[0] = nxt, b.extra[0] = cur;
            launch_inner_product_batch(ctx, b, kl.beta, lv, st);
            std::swap(cur, nxt);
        }
        for (const auto &grp : kv->res_groups) {
            if (!reduce) break;                                  // scores of a query group: the residues stay apart
            CMCHK(moddown_second_keep(ctx, cur, lv, tmp, st));
            CMCHK(ks_raise(ctx, tmp + ln, lv, digits, st));
            IpBatch b;
            b.nz = 1, b.nsum = (int)grp.size();
            for (int r = 0; r < b.nsum; r++) {
                const u64 gal = rot_g(kv, grp[r]);
                b.it[r].dig = digits, b.it[r].key = find_key(evk, gal), b.it[r].g = (unsigned)gal;
                b.it[r].c0 = cur, b.it[r].c0_ext = 1;
            }
            b.out[0] = nxt, b.extra[0] = cur;
            launch_inner_product_batch(ctx, b, kl.beta, lv, st);
            std::swap(cur, nxt);
        }
        CMCHK(moddown_into(ctx, cur, lv, nullptr, 0, 0, tmp, nullptr, st));
        CMCHK(rescale_into(ctx, tmp, 2, lv, out->dev, st));
        out->level = lv - 1, out->ncomp = 2;
        out->scale = in->scale * kv->scale / (double)ctx->mod[lv];
        RETURN_LAUNCH_STATUS();
    }
    u64 *acc = inner + (size_t)(kv->r_o - 1) * ctw;
    for (int g = kv->r_o - 2; g >= 0; g--) {
        u64 gg = rot_g(kv, kv->r_i * Ht);
        u64 *nxt = inner + (size_t)g * ctw;                      // inner_g + Rot(acc), written over inner_g
        CMCHK(rotate_into(ctx, find_key(evk, gg), acc, lv, gg, nxt, st, nxt));
        acc = nxt;
    }
    CMCHK(rescale_into(ctx, acc, 2, lv, R, st));
    for (int l = 0; l < ilog2(kv->t) && reduce; l++) {
        u64 g = rot_g(kv, 1 << l);
        CMCHK(rotate_into(ctx, find_key(evk, g), R, lv - 1, g, tmp, st, R));
        std::swap(R, tmp);
    }
    HIPCHK(hipMemcpyAsync(out->dev, R, 2 * (size_t)lv * n * 8, hipMemcpyDeviceToDevice, st));
    out->level = lv - 1, out->ncomp = 2;
    out->scale = in->scale * kv->scale / (double)ctx->mod[lv];
    RETURN_LAUNCH_STATUS();
}

extern "C" cm_status cm_vmm_kv(cm_ctx *ctx, const cm_evk *evk, const cm_kv *kv, int32_t which, const cm_ct *in,
                               cm_ct *out, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !kv || kv->ctx != ctx || !in || !in->dev || !out || !out->dev || in->ncomp != 2 || !evk_fits(ctx, evk)) return CM_E_INVAL;
    if (in->level != kv->level) return CM_E_LEVEL;
    CM_TRY
    if ((which == CM_QK || which == CM_QK_GROUP) && kv->indexed)
        return kv_sv(ctx, evk, kv, in, out, (hipStream_t)stream, false, kv->d_x, which == CM_QK);
    if (which == CM_QK || which == CM_QK_GROUP) return kv_qk(ctx, evk, kv, in, out, (hipStream_t)stream, which == CM_QK);
    if (which == CM_SV || which == CM_SV_GROUP)
        return kv_sv(ctx, evk, kv, in, out, (hipStream_t)stream, which == CM_SV, kv->d_v, false);
    return CM_E_INVAL;
    CM_CATCH
}

// ---- grouped-query attention against a cache that stores every KV head once ----------------------------------------
// The cache is the layout of Sec. 5.3 for the Hkv KV heads (t_kv tokens per K ciphertext); the query and the attention
// output use the layout for H = G Hkv heads (t = t_kv / G) with head h = hk G + g, whose slot (e, h, tau) is slot
// (e, hk, g t + tau) of the cache layout.  A query head meets all t_kv token residues of its KV head in G passes: in
// pass delta the replicated query is moved by the inner rotation (Sec. 5.4) of delta t residues and multiplied into the
// cache without further replication (CM_QK_GROUP); scores V runs per pass without the sum over the residues
// (CM_SV_GROUP), is moved back by (G - delta) t residues, the passes are added and the t residues of a run summed.
struct cm_gqa {
    cm_ctx *ctx = nullptr;
    int G = 1, t = 1, t_kv = 1, level = 0;       // level of the cache
    std::vector<cm_rope *> fwd, back;            // inner rotations by delta t at level+1 / level-1, delta = 1 .. G-1
    u64 *d_work = nullptr;                       // six ciphertexts of level+2 limbs
};
extern "C" void cm_gqa_destroy(cm_gqa *g) {
    if (!g) return;
    for (cm_rope *r : g->fwd) cm_rope_destroy(r);
    for (cm_rope *r : g->back) cm_rope_destroy(r);
    hipFree(g->d_work);
    delete g;
}
extern "C" cm_status cm_gqa_create(cm_ctx *ctx, const cm_kv *kv, int32_t group, const int64_t *coeffs, cm_gqa **out) {
    if (!ctx || !kv || kv->ctx != ctx || !out || group < 1) return CM_E_INVAL;
    if (!pow2(group) || kv->t % group) return CM_E_LAYOUT;
    if (kv->level + 1 > ctx->L || kv->level < 2) return CM_E_LEVEL;
    cm_gqa *g = new (std::nothrow) cm_gqa();
    if (!g) return CM_E_NOMEM;
    try {
        g->ctx = ctx, g->G = group, g->t_kv = kv->t, g->t = kv->t / group, g->level = kv->level;
        const size_t n = ctx->n;
        if (hipMalloc((void **)&g->d_work, 6 * 2 * (size_t)(kv->level + 2) * n * 8) != hipSuccess) {
            cm_gqa_destroy(g);
            return CM_E_NOMEM;
        }
        for (int dir = 0; dir < 2; dir++)
            for (int delta = 1; delta < group; delta++) {
                cm_rope *r = nullptr;
                const int64_t *cf = coeffs ? coeffs + ((size_t)dir * (group - 1) + (delta - 1)) * 3 * n : nullptr;
                cm_status s = cm_inner_rot_create(ctx, kv->t, delta * g->t, dir == 0 ? kv->level + 1 : kv->level - 1, cf, &r);
                if (s != CM_OK) {
                    cm_gqa_destroy(g);
                    return s;
                }
                (dir == 0 ? g->fwd : g->back).push_back(r);
            }
    } catch (...) {
        cm_gqa_destroy(g);
        return CM_E_NOMEM;
    }
    *out = g;
    return CM_OK;
}
static std::vector<int> gqa_all_steps(const cm_gqa *g) {
    std::vector<int> s;
    for (int i = 0; i < ilog2(g->t); i++) s.push_back(-(1 << i));            // replicate the query over its run
    for (int delta = 1; delta < g->G; delta++) s.push_back(-delta * g->t), s.push_back(g->t_kv - delta * g->t);   // inner rotations
    for (int l = 0; l < ilog2(g->t); l++) s.push_back(1 << l);               // sum over the residues of a run
    return s;
}
extern "C" int32_t cm_gqa_steps(const cm_gqa *g, int32_t *steps, int32_t cap) {
    if (!g) return 0;
    try {
        auto s = gqa_all_steps(g);
        for (int i = 0; i < (int)s.size() && i < cap && steps; i++) steps[i] = s[i];
        return (int32_t)s.size();
    } catch (...) {
        return 0;
    }
}
static cm_status gqa_keys(cm_ctx *ctx, const cm_evk *evk, const cm_gqa *g) {
    for (int a : gqa_all_steps(g))
        if (!find_key(evk, galois_of_step(ctx, a))) return CM_E_NOKEY;
    return CM_OK;
}
extern "C" cm_status cm_gqa_qk(cm_ctx *ctx, const cm_evk *evk, const cm_gqa *g, const cm_kv *kv, const cm_ct *q, cm_ct *scores,
                               void *stream) {
    (void)hipGetLastError();
    if (!ctx || !evk || !g || !kv || g->ctx != ctx || kv->ctx != ctx || !q || !q->dev || q->ncomp != 2 || !scores || !evk_fits(ctx, evk))
        return CM_E_INVAL;
    if (kv->t != g->t_kv || kv->level != g->level) return CM_E_LAYOUT;
    if (q->level != kv->level + 1) return CM_E_LEVEL;
    for (int d = 0; d < g->G; d++) if (!scores[d].dev) return CM_E_INVAL;
    CM_TRY
    CMCHK(gqa_keys(ctx, evk, g));
    // a cache with the key index: every pass is the scores-times-V schedule on the index (scores one level below the
    // cache); otherwise the un-replicated query-times-K of the cache's form (two levels below)
    if (kv->indexed) CMCHK(kv_sv_keys(evk, kv, false, false));
    else CMCHK(kv_qk_keys(evk, kv, false));
    hipStream_t st = (hipStream_t)stream;
    const int lq = q->level;
    const size_t n = ctx->n, ctq = 2 * (size_t)(lq + 1) * n, slot = 2 * (size_t)(kv->level + 2) * n;
    u64 *cq = g->d_work, *alt = cq + slot, *xd = alt + slot;
    HIPCHK(hipMemcpyAsync(cq, q->dev, ctq * 8, hipMemcpyDeviceToDevice, st));
    for (int i = 0; i < ilog2(g->t); i++) {
        const u64 gal = galois_of_step(ctx, -(1 << i));
        CMCHK(rotate_into(ctx, find_key(evk, gal), cq, lq, gal, alt, st, cq));      // alt = cq + Rot(cq)
        std::swap(cq, alt);
    }
    cm_ct rep{cq, lq, 2, q->scale}, x{xd, kv->level, 2, q->scale};
    for (int delta = 0; delta < g->G; delta++) {
        if (delta == 0) CMCHK(cm_level_drop(ctx, &rep, kv->level, &x, stream));
        else CMCHK(cm_rope_apply(ctx, evk, g->fwd[delta - 1], &rep, &x, stream));
        if (kv->indexed) CMCHK(kv_sv(ctx, evk, kv, &x, &scores[delta], st, false, kv->d_x, false));
        else CMCHK(kv_qk(ctx, evk, kv, &x, &scores[delta], st, false));
    }
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
extern "C" cm_status cm_gqa_sv(cm_ctx *ctx, const cm_evk *evk, const cm_gqa *g, const cm_kv *kv, const cm_ct *scores, cm_ct *out,
                               void *stream) {
    (void)hipGetLastError();
    if (!ctx || !evk || !g || !kv || g->ctx != ctx || kv->ctx != ctx || !scores || !out || !out->dev || !evk_fits(ctx, evk))
        return CM_E_INVAL;
    if (kv->t != g->t_kv || kv->level != g->level) return CM_E_LAYOUT;
    for (int d = 0; d < g->G; d++) {
        if (!scores[d].dev || scores[d].ncomp != 2) return CM_E_INVAL;
        if (scores[d].level != kv->level) return CM_E_LEVEL;
        if (fabs(scores[d].scale / scores[0].scale - 1) > 1e-9) return CM_E_SCALE;
    }
    CM_TRY
    CMCHK(gqa_keys(ctx, evk, g));
    CMCHK(kv_sv_keys(evk, kv, false, false));
    hipStream_t st = (hipStream_t)stream;
    const int lv = kv->level, lo = lv - 2;
    const size_t n = ctx->n, slot = 2 * (size_t)(lv + 2) * n;
    u64 *pd = g->d_work, *md = pd + slot, *acc = md + slot, *alt = acc + slot;
    cm_ct part{pd, lv - 1, 2, 0.0}, moved{md, lo, 2, 0.0};
    for (int delta = 0; delta < g->G; delta++) {
        CMCHK(kv_sv(ctx, evk, kv, &scores[delta], &part, st, false, kv->d_v, false));
        const int back = (g->G - delta) % g->G;
        cm_ct dst{delta == 0 ? acc : md, lo, 2, 0.0};
        if (back == 0) CMCHK(cm_level_drop(ctx, &part, lo, &dst, stream));
        else CMCHK(cm_rope_apply(ctx, evk, g->back[back - 1], &part, &dst, stream));
        if (delta) launch_add(ctx, acc, acc, md, 2, lo + 1, st);
        moved.scale = dst.scale;
    }
    for (int l = 0; l < ilog2(g->t); l++) {
        const u64 gal = galois_of_step(ctx, 1 << l);
        CMCHK(rotate_into(ctx, find_key(evk, gal), acc, lo, gal, alt, st, acc));
        std::swap(acc, alt);
    }
    HIPCHK(hipMemcpyAsync(out->dev, acc, 2 * (size_t)(lo + 1) * n * 8, hipMemcpyDeviceToDevice, st));
    out->level = lo, out->ncomp = 2, out->scale = moved.scale;
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
