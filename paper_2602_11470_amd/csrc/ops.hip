// C ABI: keys, encryption, the ciphertext operations of Sec. 2.1 and hybrid key switching.
#include <math.h>
#include <string.h>

#include <algorithm>

#include "kernels.h"

// stream identifiers of the counter-based generator
// The seed a call receives is public (the uniform halves are its streams); the error streams are keyed by that seed
// XOR the secret key's `noise`, the key of stream ST_NOISE under the secret key's own seed.
enum { ST_SECRET = 1, ST_EVK_A = 2, ST_EVK_E = 3, ST_ENC_A = 4, ST_ENC_E = 5, ST_NOISE = 6 };
static inline u64 stream_id(u64 purpose, u64 ident, u64 digit, u64 limb) {
    return (purpose << 56) | (ident << 16) | (digit << 8) | limb;
}

// ---- arena ------------------------------------------------------------------------------------
struct Arena {
    u64 *ksin, *digits, *u, *conv, *tmp[3], *misc, *bu, *bconv;
};
static Arena arena_of(const cm_ctx *ctx) {
    const size_t n = ctx->n, q = ctx->L + 1, ext = ctx->L + 1 + ctx->K;
    const size_t beta = (ctx->L + ctx->alpha) / ctx->alpha;
    Arena a;
    u64 *p = ctx->arena;
    a.ksin = p, p += q * n;
    a.digits = p, p += beta * ext * n;
    a.u = p, p += 2 * ext * n;
    a.conv = p, p += 2 * q * n;
    for (int i = 0; i < 3; i++) a.tmp[i] = p, p += 3 * q * n;
    a.misc = p, p += 4 * n;
    a.bu = p, p += 2 * (size_t)CM_KS_BATCH * 2 * ext * n;      // two batches in flight
    a.bconv = p;
    return a;
}

// device copy of a host table (nullptr for an empty one); failure raises std::bad_alloc, caught at the C boundary
template <class T>
static T *up(const std::vector<T> &v) {
    T *d = nullptr;
    if (v.empty()) return nullptr;
    if (hipMalloc((void **)&d, v.size() * sizeof(T)) != hipSuccess) throw std::bad_alloc();
    if (hipMemcpy(d, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) {
        hipFree(d);
        throw std::bad_alloc();
    }
    return d;
}
// The synchronous calls (keys, encode, encrypt, decrypt, decode, exports) work on the null stream and share the
// context's arena with the enqueueing calls: they first wait for everything the device still has in flight, so that
// work pending on a caller's non-blocking stream cannot overlap them.
static cm_status sync_begin() {
    HIPCHK(hipDeviceSynchronize());
    return CM_OK;
}

struct KsLevelFull : KsLevel {
    int *d_q_mods3 = nullptr;   // 0..level repeated three times
    int *d_last_mods = nullptr; // level, repeated for up to RESCALE_MAX_COMPS components
    int *d_red_mods = nullptr;  // 0..level-1, repeated likewise
    int *d_red_src = nullptr;   // the component each of those limbs belongs to (its row in the stacked last limbs)
    bool last_fits = false;     // the last modulus is below twice every other one (and below 2^52): its residues can enter
                                // the other limbs' transforms as they are
    int *d_last_rows = nullptr; // rows c*(level+1)+level of stacked components
    int *d_bsp_rows = nullptr, *d_bsp_mods = nullptr;   // special rows of CM_KS_BATCH stacked [2][ext] blocks
    int *d_bsp1_rows = nullptr;                         // those of the second components only
    int *d_sp1_rows = nullptr;                          // special rows of the second component of one [2][ext] block
    ConvDev *d_moddown0 = nullptr;                      // the ModDown conversion reading its K input limbs from rows 0..K-1
    int *d_bq_mods = nullptr;                           // 0..level repeated 2*CM_KS_BATCH times
    std::vector<int> h_ntt_rows, h_ntt_mods;            // host copies of d_ntt_rows / d_ntt_mods
    ConvDev *d_modup = nullptr; // one table per digit
    ConvDev *d_moddown = nullptr;
    int modup_max_nt = 0;
};

#define RESCALE_MAX_COMPS (2 * CM_KS_BATCH)
#define IDX_CHUNK_U64 128
static ConvDev conv_dev(const cm_ctx *ctx, const ConvTable &t, const std::vector<int> &in_rows,
                        const std::vector<int> &out_rows) {
    ConvDev d;
    memset(&d, 0, sizeof(d));
    d.ns = t.ns, d.nt = t.nt;
    for (int m = 0; m < t.ns; m++) {
        d.src_mod[m] = t.src[m], d.in_rows[m] = in_rows[m];
        d.inv_hat[m] = t.inv_hat[m], d.inv_hat_sh[m] = t.inv_hat_sh[m];
        d.src_q[m] = ctx->mod[t.src[m]];
    }
    for (int r = 0; r < t.nt; r++) {
        d.dst_mod[r] = t.dst[r], d.out_rows[r] = out_rows[r];
        d.dst_q[r] = ctx->modc[t.dst[r]].q, d.dst_qinv[r] = ctx->modc[t.dst[r]].qinv;
    }
    for (size_t i = 0; i < t.hat_mont.size(); i++) d.hat_mont[i] = t.hat_mont[i];
    return d;
}
static std::map<std::pair<cm_ctx *, int>, KsLevelFull> g_ks;

static void free_ks(KsLevelFull &k) {
    hipFree(k.d_modup); hipFree(k.d_moddown); hipFree(k.d_bsp_rows); hipFree(k.d_bsp1_rows); hipFree(k.d_sp1_rows); hipFree(k.d_moddown0); hipFree(k.d_bsp_mods); hipFree(k.d_bq_mods);
    hipFree(k.d_last_rows);
    hipFree(k.d_ntt_rows); hipFree(k.d_ntt_mods); hipFree(k.d_sp_rows); hipFree(k.d_sp_mods);
    hipFree(k.d_q_rows); hipFree(k.d_q_mods3); hipFree(k.d_last_mods); hipFree(k.d_red_mods); hipFree(k.d_red_src);
}
static void build_ks(cm_ctx *ctx, int level, KsLevelFull &k);
static const KsLevelFull &ks_level_full(cm_ctx *ctx, int level) {
    auto key = std::make_pair(ctx, level);
    auto it = g_ks.find(key);
    if (it != g_ks.end()) return it->second;
    KsLevelFull k;
    try {
        build_ks(ctx, level, k);
        return g_ks[key] = k;
    } catch (...) {              // a table did not fit: nothing half-built is kept
        free_ks(k);
        g_ks.erase(key);
        throw;
    }
}
static void build_ks(cm_ctx *ctx, int level, KsLevelFull &k) {
    k.level = level;
    k.ext = level + 1 + ctx->K;
    auto digs = digits_at(ctx, level);
    k.beta = (int)digs.size();
    const auto &tabs = get_modup(ctx, level);
    std::vector<int> ntt_rows, ntt_mods;
    std::vector<ConvDev> mu;
    for (int j = 0; j < k.beta; j++) {
        std::vector<int> out_rows;
        for (int idx : tabs[j].dst) {
            int row = idx <= level ? idx : level + 1 + (idx - ctx->L - 1);
            out_rows.push_back(row);
            ntt_rows.push_back(j * k.ext + row);
            ntt_mods.push_back(idx);
        }
        mu.push_back(conv_dev(ctx, tabs[j], digs[j], out_rows));
        k.modup_max_nt = std::max(k.modup_max_nt, tabs[j].nt);
    }
    k.d_modup = up(mu);
    {
        // Transform the converted limbs modulus by modulus rather than digit by digit: the limbs that
        // share a twiddle table are then adjacent in the launch and the table is reused from L2
        // instead of being refetched by every XCD for every digit.
        std::vector<int> order(ntt_rows.size());
        for (size_t i = 0; i < order.size(); i++) order[i] = (int)i;
        // The limbs under the 60-bit primes go first: their integer butterflies take about twice the instructions of the
        // FP64 ones, and a launch that ends on them has a long tail of its slowest workgroups.
        auto slow = [&](int i) { return ctx->mod[ntt_mods[i]] >= (1ULL << 50) ? 0 : 1; };
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
            return slow(a) != slow(b) ? slow(a) < slow(b) : ntt_mods[a] < ntt_mods[b];
        });
        std::vector<int> r2, m2;
        for (int i : order) r2.push_back(ntt_rows[i]), m2.push_back(ntt_mods[i]);
        ntt_rows.swap(r2), ntt_mods.swap(m2);
    }
    k.d_ntt_rows = up(ntt_rows);
    k.d_ntt_mods = up(ntt_mods);
    k.h_ntt_rows = ntt_rows, k.h_ntt_mods = ntt_mods;
    k.n_ntt = (int)ntt_rows.size();
    std::vector<int> sp_rows, sp_mods, q_rows, q3, last(RESCALE_MAX_COMPS, level), red;
    for (int c = 0; c < 2; c++)
        for (int s = 0; s < ctx->K; s++) {
            sp_rows.push_back(c * k.ext + level + 1 + s);
            sp_mods.push_back(ctx->L + 1 + s);
        }
    for (int i = 0; i <= level; i++) q_rows.push_back(i);
    for (int c = 0; c < 3; c++)
        for (int i = 0; i <= level; i++) q3.push_back(i);
    std::vector<int> red_src;
    for (int c = 0; c < RESCALE_MAX_COMPS; c++)
        for (int i = 0; i < level; i++) red.push_back(i), red_src.push_back(c);
    if (red.empty()) red.push_back(0), red_src.push_back(0);
    k.last_fits = ctx->mod[level] < (1ULL << 52);
    for (int i = 0; i < level; i++) k.last_fits = k.last_fits && ctx->mod[level] < 2 * ctx->mod[i];
    k.d_sp_rows = up(sp_rows);
    k.d_sp_mods = up(sp_mods);
    k.d_q_rows = up(q_rows);
    k.d_q_mods3 = up(q3);
    k.d_last_mods = up(last);
    k.d_red_mods = up(red);
    k.d_red_src = up(red_src);
    {
        std::vector<int> br, bm, bq;
        for (int r = 0; r < CM_KS_BATCH; r++)
            for (int c = 0; c < 2; c++) {
                for (int sp = 0; sp < ctx->K; sp++) {
                    br.push_back((r * 2 + c) * k.ext + level + 1 + sp);
                    bm.push_back(ctx->L + 1 + sp);
                }
                for (int i = 0; i <= level; i++) bq.push_back(i);
            }
        k.d_bsp_rows = up(br), k.d_bsp_mods = up(bm), k.d_bq_mods = up(bq);
        std::vector<int> b1;
        for (int r = 0; r < CM_KS_BATCH; r++)
            for (int sp = 0; sp < ctx->K; sp++) b1.push_back((r * 2 + 1) * k.ext + level + 1 + sp);
        k.d_bsp1_rows = up(b1);
    }
    {
        std::vector<int> lr;
        for (int c = 0; c < RESCALE_MAX_COMPS; c++) lr.push_back(c * (level + 1) + level);
        k.d_last_rows = up(lr);
    }
    {
        std::vector<int> sp_in;
        for (int s = 0; s < ctx->K; s++) sp_in.push_back(level + 1 + s);
        std::vector<ConvDev> md(1, conv_dev(ctx, get_moddown(ctx, level), sp_in, q_rows));
        k.d_moddown = up(md);
        std::vector<int> sp0, sp1;
        for (int s = 0; s < ctx->K; s++) sp0.push_back(s), sp1.push_back(k.ext + level + 1 + s);
        std::vector<ConvDev> md0(1, conv_dev(ctx, get_moddown(ctx, level), sp0, q_rows));
        k.d_moddown0 = up(md0);
        k.d_sp1_rows = up(sp1);
    }
    get_pinv(ctx, level);
    get_qlinv(ctx, level);
}
const KsLevel &ks_level(cm_ctx *ctx, int level) { return ks_level_full(ctx, level); }

static void drop_ks_levels(cm_ctx *ctx) {
    for (auto it = g_ks.begin(); it != g_ks.end();) {
        if (it->first.first != ctx) { ++it; continue; }
        free_ks(it->second);
        it = g_ks.erase(it);
    }
}
// called from cm_ctx_destroy's translation unit through this hook
void cm_ops_forget_ctx(cm_ctx *ctx) { drop_ks_levels(ctx); }

static bool ct_ok(const cm_ctx *ctx, const cm_ct *c) {
    return c && c->dev && c->level >= 0 && c->level <= ctx->L && (c->ncomp == 2 || c->ncomp == 3);
}
static bool same_scale(double a, double b) { return fabs(a / b - 1.0) < 1e-9; }

// ---- hybrid key switching -------------------------------------------------------------------------
cm_status ks_raise(cm_ctx *ctx, const u64 *d, int level, u64 *digits, hipStream_t st, u64 g) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n;
    // coefficient-domain copy of d (out of place), then all digits in one conversion launch; a
    // digit's own limbs are copied from d itself, which is already in the evaluation domain
    launch_ntt_src(ctx, A.ksin, nullptr, d, nullptr, iota_idx(ctx), level + 1, true, st, g);
    launch_base_conv(ctx, k.d_modup, k.beta, 1, k.modup_max_nt, digits, A.ksin, 0, (size_t)k.ext * n, d, g, st);
    launch_ntt_rows(ctx, digits, k.d_ntt_rows, k.d_ntt_mods, k.n_ntt, false, st);
    return CM_OK;
}

cm_status moddown_into(cm_ctx *ctx, u64 *u, int level, const u64 *addend, int addend_comps, u64 g, u64 *out,
                       const u64 *accum, hipStream_t st) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n;
    if (!addend) addend_comps = 0, g = 0;
    launch_ntt_rows(ctx, u, k.d_sp_rows, k.d_sp_mods, 2 * ctx->K, true, st);
    launch_base_conv(ctx, k.d_moddown, 2, 0, level + 1, A.conv, u, (size_t)k.ext * n, (size_t)(level + 1) * n, nullptr, 0, st);
    if (ctx->n == 65536) {
        FinishBatch fb;
        fb.items = 1, fb.level = level, fb.ext = k.ext, fb.addend_comps = addend_comps;
        fb.u[0] = u, fb.out[0] = out, fb.accum[0] = accum, fb.g[0] = (unsigned)g;
        fb.addend[0] = addend, fb.pinv = get_pinv(ctx, level);
        launch_ntt_fwd_finish(ctx, A.conv, k.d_q_mods3, fb, st);
        return CM_OK;
    }
    launch_ntt(ctx, A.conv, k.d_q_mods3, 2 * (level + 1), false, st);
    launch_moddown_finish(ctx, out, u, A.conv, get_pinv(ctx, level), addend, addend_comps, level, g, accum, st);
    return CM_OK;
}

cm_status ks_apply(cm_ctx *ctx, const u64 *digits, const u64 *evk, int level, u64 g, const u64 *addend,
                   int addend_comps, u64 *out, hipStream_t st, const u64 *accum) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    launch_inner_product(ctx, A.u, A.u + (size_t)k.ext * ctx->n, digits, evk, k.beta, level, g, st);
    return moddown_into(ctx, A.u, level, addend, addend_comps, g, out, accum, st);
}
// inverse of the odd g modulo the power of two 2n (Newton's iteration doubles the correct low bits)
static unsigned galois_inverse(const cm_ctx *ctx, u64 g) {
    const u64 two_n = 2 * (u64)ctx->n;
    g %= two_n;
    u64 x = g;
    for (int it = 0; it < 6; it++) x = (x * (2 - g * x)) % two_n;
    return (unsigned)x;
}
cm_status ks_apply_many_raised(cm_ctx *ctx, const u64 *digits, int level, int cnt, const u64 *const *keys,
                               const u64 *gs, const u64 *in, u64 *const *raised, hipStream_t st, bool in_ext) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    if (k.beta <= 8) {
        // one digit array, many keys: the lanes keep the digits and walk over the keys (inverse Galois maps)
        for (int base = 0; base < cnt; base += IP_FAN_MAX) {
            IpFan f;
            f.n = cnt - base < IP_FAN_MAX ? cnt - base : IP_FAN_MAX;
            for (int r = 0; r < f.n; r++) {
                f.key[r] = keys[base + r], f.out[r] = raised[base + r];
                f.ginv[r] = galois_inverse(ctx, gs[base + r]);
            }
            launch_inner_product_fanout(ctx, f, digits, in, in_ext, k.beta, level, st);
        }
        return CM_OK;
    }
    for (int base = 0; base < cnt; base += IP_MAX_ITEMS) {
        IpBatch b;
        b.nz = cnt - base < IP_MAX_ITEMS ? cnt - base : IP_MAX_ITEMS, b.nsum = 1;
        for (int r = 0; r < b.nz; r++) {
            b.it[r].dig = digits, b.it[r].key = keys[base + r], b.it[r].c0 = in, b.it[r].g = (unsigned)gs[base + r];
            b.it[r].c0_ext = in_ext ? 1 : 0;
            b.out[r] = raised[base + r], b.extra[r] = nullptr;
        }
        launch_inner_product_batch(ctx, b, k.beta, level, st);
    }
    return CM_OK;
}
u64 *arena_digits(const cm_ctx *ctx) { return arena_of(ctx).digits; }
u64 *arena_batch_sums(const cm_ctx *ctx) { return arena_of(ctx).bu; }

// ModDown of m <= CM_KS_BATCH stacked sums bu[r][2][ext][n] in one batch of launches:
// outs[r] = ModDown(bu[r]) (+ perm_{gs[r]}(addends[r]) on the first addend_comps components) (+ accums[r])
static void moddown_batch(cm_ctx *ctx, const KsLevelFull &k, u64 *bu, int m, const u64 *const *addends, int addend_comps,
                          const u64 *gs, const u64 *const *accums, u64 *const *outs, hipStream_t st) {
    Arena A = arena_of(ctx);
    const int level = k.level;
    const size_t n = ctx->n, ublk = 2 * (size_t)k.ext * n, cblk = 2 * (size_t)(level + 1) * n;
    launch_ntt_rows(ctx, bu, k.d_bsp_rows, k.d_bsp_mods, m * 2 * ctx->K, true, st);
    launch_base_conv(ctx, k.d_moddown, 2 * m, 0, level + 1, A.bconv, bu, (size_t)k.ext * n, (size_t)(level + 1) * n, nullptr,
                     0, st);
    auto add_of = [&](int r) { return addends ? addends[r] : nullptr; };
    auto acc_of = [&](int r) { return accums ? accums[r] : nullptr; };
    if (ctx->n == 65536) {
        FinishBatch fb;
        fb.items = m, fb.level = level, fb.ext = k.ext, fb.addend_comps = addends ? addend_comps : 0;
        for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr;
        for (int r = 0; r < m; r++) {
            fb.u[r] = bu + r * ublk, fb.out[r] = outs[r], fb.accum[r] = acc_of(r), fb.addend[r] = add_of(r);
            fb.g[r] = add_of(r) && gs ? (unsigned)gs[r] : 0;
        }
        fb.pinv = get_pinv(ctx, level);
        launch_ntt_fwd_finish(ctx, A.bconv, k.d_bq_mods, fb, st);
    } else {
        launch_ntt(ctx, A.bconv, k.d_bq_mods, m * 2 * (level + 1), false, st);
        for (int r = 0; r < m; r++)
            launch_moddown_finish(ctx, outs[r], bu + r * ublk, A.bconv + r * cblk, get_pinv(ctx, level), add_of(r),
                                  add_of(r) ? addend_comps : 0, level, add_of(r) && gs ? gs[r] : 0, acc_of(r), st);
    }
}
cm_status moddown_batch_into(cm_ctx *ctx, u64 *us, int level, int m, const u64 *const *addends, int addend_comps, u64 g,
                             const u64 *const *accums, u64 *const *outs, hipStream_t st) {
    if (m < 1 || m > CM_KS_BATCH) return CM_E_INVAL;
    u64 gs[CM_KS_BATCH];
    for (int r = 0; r < m; r++) gs[r] = g;
    moddown_batch(ctx, ks_level_full(ctx, level), us, m, addends, addend_comps, gs, accums, outs, st);
    return CM_OK;
}
cm_status moddown_many(cm_ctx *ctx, u64 *us, int level, int cnt, u64 *const *outs, hipStream_t st) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    const size_t ublk = 2 * (size_t)k.ext * ctx->n;
    for (int base = 0; base < cnt; base += CM_KS_BATCH) {
        const int m = cnt - base < CM_KS_BATCH ? cnt - base : CM_KS_BATCH;
        moddown_batch(ctx, k, us + base * ublk, m, nullptr, 0, nullptr, nullptr, outs + base, st);
    }
    return CM_OK;
}

cm_status moddown_many_second(cm_ctx *ctx, u64 *us, int level, int cnt, u64 *const *outs, hipStream_t st) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n, ublk = 2 * (size_t)k.ext * n;
    for (int base = 0; base < cnt; base += CM_KS_BATCH) {
        const int m = cnt - base < CM_KS_BATCH ? cnt - base : CM_KS_BATCH;
        u64 *bu = us + base * ublk;
        // special limbs of the second components to the coefficient domain, converted to q_0..q_level, transformed,
        // and the tail (u - conv) P^{-1} fused into the last pass of that transform
        launch_ntt_rows(ctx, bu, k.d_bsp1_rows, k.d_bsp_mods, m * ctx->K, true, st);
        launch_base_conv(ctx, k.d_moddown, m, 0, level + 1, A.bconv, bu + (size_t)k.ext * n, ublk, (size_t)(level + 1) * n,
                         nullptr, 0, st);
        if (ctx->n != 65536) {                              // no fused tail at the small ring sizes
            launch_ntt(ctx, A.bconv, k.d_bq_mods, m * (level + 1), false, st);
            for (int r = 0; r < m; r++)
                launch_moddown_finish(ctx, outs[base + r] + (size_t)(level + 1) * n, bu + r * ublk + (size_t)k.ext * n,
                                      A.bconv + (size_t)r * (level + 1) * n, get_pinv(ctx, level), nullptr, 0, level, 0,
                                      nullptr, st, 1);
            continue;
        }
        FinishBatch fb;
        fb.items = m, fb.level = level, fb.ext = k.ext, fb.addend_comps = 0, fb.ncomp = 1, fb.comp0 = 1;
        for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr, fb.u[r] = nullptr, fb.out[r] = nullptr, fb.g[r] = 0;
        for (int r = 0; r < m; r++) fb.u[r] = bu + r * ublk, fb.out[r] = outs[base + r];
        fb.pinv = get_pinv(ctx, level);
        launch_ntt_fwd_finish(ctx, A.bconv, k.d_bq_mods, fb, st);
    }
    return CM_OK;
}

cm_status moddown_second_keep(cm_ctx *ctx, const u64 *R, int level, u64 *out, hipStream_t st) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n;
    // the K special limbs of the second component, to the coefficient domain in a buffer of their own
    launch_ntt_src(ctx, A.tmp[0], nullptr, R, k.d_sp1_rows, k.d_sp_mods, ctx->K, true, st, 0);
    launch_base_conv(ctx, k.d_moddown0, 1, 0, level + 1, A.bconv, A.tmp[0], 0, 0, nullptr, 0, st);
    if (ctx->n != 65536) {
        launch_ntt(ctx, A.bconv, k.d_bq_mods, level + 1, false, st);
        launch_moddown_finish(ctx, out + (size_t)(level + 1) * n, R + (size_t)k.ext * n, A.bconv, get_pinv(ctx, level), nullptr, 0,
                              level, 0, nullptr, st, 1);
        return CM_OK;
    }
    FinishBatch fb;
    fb.items = 1, fb.level = level, fb.ext = k.ext, fb.addend_comps = 0, fb.ncomp = 1, fb.comp0 = 1;
    for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr, fb.u[r] = nullptr, fb.out[r] = nullptr, fb.g[r] = 0;
    fb.u[0] = R, fb.out[0] = out, fb.pinv = get_pinv(ctx, level);
    launch_ntt_fwd_finish(ctx, A.bconv, k.d_bq_mods, fb, st);
    return CM_OK;
}

cm_status moddown_second_keep_many(cm_ctx *ctx, const u64 *Rs, int level, int m, u64 *const *outs, hipStream_t st) {
    if (m < 1 || m > CM_KS_BATCH) return CM_E_INVAL;
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n, ublk = 2 * (size_t)k.ext * n;
    // the K special limbs of every second component, to the coefficient domain in a buffer of their own
    // (the three temporaries of the arena are contiguous: 9 (L+1) limbs, room for CM_KS_BATCH * K)
    launch_ntt_src(ctx, A.tmp[0], nullptr, Rs, k.d_bsp1_rows, k.d_bsp_mods, m * ctx->K, true, st, 0);
    launch_base_conv(ctx, k.d_moddown0, m, 0, level + 1, A.bconv, A.tmp[0], (size_t)ctx->K * n, (size_t)(level + 1) * n, nullptr,
                     0, st);
    if (ctx->n != 65536) {
        launch_ntt(ctx, A.bconv, k.d_bq_mods, m * (level + 1), false, st);
        for (int r = 0; r < m; r++)
            launch_moddown_finish(ctx, outs[r] + (size_t)(level + 1) * n, Rs + r * ublk + (size_t)k.ext * n,
                                  A.bconv + (size_t)r * (level + 1) * n, get_pinv(ctx, level), nullptr, 0, level, 0, nullptr,
                                  st, 1);
        return CM_OK;
    }
    FinishBatch fb;
    fb.items = m, fb.level = level, fb.ext = k.ext, fb.addend_comps = 0, fb.ncomp = 1, fb.comp0 = 1;
    for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr, fb.u[r] = nullptr, fb.out[r] = nullptr, fb.g[r] = 0;
    for (int r = 0; r < m; r++) fb.u[r] = Rs + r * ublk, fb.out[r] = outs[r];
    fb.pinv = get_pinv(ctx, level);
    launch_ntt_fwd_finish(ctx, A.bconv, k.d_bq_mods, fb, st);
    return CM_OK;
}

cm_status ks_many_tables_create(cm_ctx *ctx, int level, int cnt, KsManyTables *t, int ncomp, int comp) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    std::vector<int> src_rows, in_mods, rows, mods;
    t->ncomp = ncomp, t->comp = comp;
    for (int c = 0; c < cnt; c++) {
        for (int l = 0; l <= level; l++) src_rows.push_back((c * ncomp + comp) * (level + 1) + l), in_mods.push_back(l);
        for (size_t i = 0; i < k.h_ntt_rows.size(); i++)
            rows.push_back(c * k.beta * k.ext + k.h_ntt_rows[i]), mods.push_back(k.h_ntt_mods[i]);
    }
    t->cnt = cnt, t->level = level, t->n_ntt = (int)k.h_ntt_rows.size();
    try {
        t->d_src_rows = up(src_rows), t->d_in_mods = up(in_mods), t->d_ntt_rows = up(rows), t->d_ntt_mods = up(mods);
    } catch (const std::bad_alloc &) {
        ks_many_tables_destroy(t);
        return CM_E_NOMEM;
    }
    return CM_OK;
}
void ks_many_tables_destroy(KsManyTables *t) {
    hipFree(t->d_src_rows); hipFree(t->d_in_mods); hipFree(t->d_ntt_rows); hipFree(t->d_ntt_mods);
    *t = KsManyTables();
}
cm_status ks_raise_many(cm_ctx *ctx, const KsManyTables &t, const u64 *cts, u64 *ksin, u64 *digits, hipStream_t st, int m,
                        u64 g) {
    if (m < 0) m = t.cnt;
    if (m == 0) return CM_OK;
    if (m > t.cnt) return CM_E_INVAL;
    const KsLevelFull &k = ks_level_full(ctx, t.level);
    const size_t n = ctx->n, ln = (size_t)(t.level + 1) * n;
    // the tables list the items in order, so the first m items are a prefix of every table
    launch_ntt_src(ctx, ksin, nullptr, cts, t.d_src_rows, t.d_in_mods, m * (t.level + 1), true, st, g);
    launch_base_conv(ctx, k.d_modup, m * k.beta, 1, k.modup_max_nt, digits, ksin, ln, (size_t)k.ext * n,
                     cts + (size_t)t.comp * ln, g, st, k.beta, k.beta, (size_t)t.ncomp * ln);
    launch_ntt_rows(ctx, digits, t.d_ntt_rows, t.d_ntt_mods, m * t.n_ntt, false, st);
    return CM_OK;
}

// cnt hoisted rotations of one ciphertext `in` ([2][level+1][n]) whose raised digits are given:
// outs[r] = ModDown(sum_j perm_{g_r}(digits_j) * key_r) + perm_{g_r}(in.c0).  The ModDown of up to
// CM_KS_BATCH rotations runs as one batch so that its transforms and conversions fill the machine.
cm_status ks_apply_many(cm_ctx *ctx, const u64 *digits, int level, int cnt, const u64 *const *keys, const u64 *gs,
                        const u64 *in, u64 *const *outs, hipStream_t st) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    const size_t n = ctx->n, ublk = 2 * (size_t)k.ext * n, cblk = 2 * (size_t)(level + 1) * n;
    const size_t bufw = (size_t)CM_KS_BATCH * ublk;
    // batch by batch: the inner products of CM_KS_BATCH rotations (the digits read once for all of them), then their
    // ModDown as one batch of launches; two result buffers alternate
    (void)cblk;
    for (int base = 0, b = 0; base < cnt; base += CM_KS_BATCH, b++) {
        const int m = cnt - base < CM_KS_BATCH ? cnt - base : CM_KS_BATCH;
        u64 *bu = A.bu + (b & 1) * bufw;
        if (k.beta <= 8) {
            IpFan f;
            f.n = m;
            for (int r = 0; r < m; r++) f.key[r] = keys[base + r], f.out[r] = bu + r * ublk, f.ginv[r] = galois_inverse(ctx, gs[base + r]);
            launch_inner_product_fanout(ctx, f, digits, nullptr, false, k.beta, level, st);
        } else {
            for (int r = 0; r < m; r++)
                launch_inner_product(ctx, bu + r * ublk, bu + r * ublk + (size_t)k.ext * n, digits, keys[base + r],
                                     k.beta, level, gs[base + r], st);
        }
        const u64 *adds[CM_KS_BATCH];
        for (int r = 0; r < m; r++) adds[r] = in;
        moddown_batch(ctx, k, bu, m, adds, 1, gs + base, nullptr, outs + base, st);
    }
    return CM_OK;
}

const u64 *find_key(const cm_evk *evk, u64 g) {
    auto it = evk->keys.find(g);
    return it == evk->keys.end() ? nullptr : it->second.d;
}
bool evk_fits(const cm_ctx *ctx, const cm_evk *evk) { return evk && evk->stored_a == ctx->evk_stored_a; }

extern "C" cm_status cm_keyswitch(cm_ctx *ctx, const cm_evk *evk, int32_t step, int32_t relin, const uint64_t *d,
                                  int32_t level, uint64_t *ks0, uint64_t *ks1, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !d || !ks0 || !ks1 || level < 0 || level > ctx->L || !evk_fits(ctx, evk)) return CM_E_INVAL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    const u64 *key = find_key(evk, relin ? 0 : galois_of_step(ctx, step));
    if (!key) return CM_E_NOKEY;
    Arena A = arena_of(ctx);
    CMCHK(ks_raise(ctx, (const u64 *)d, level, A.digits, st));
    CMCHK(ks_apply(ctx, A.digits, key, level, 0, nullptr, 0, A.tmp[0], st));
    size_t bytes = (size_t)(level + 1) * ctx->n * 8;
    HIPCHK(hipMemcpyAsync(ks0, A.tmp[0], bytes, hipMemcpyDeviceToDevice, st));
    HIPCHK(hipMemcpyAsync(ks1, A.tmp[0] + (size_t)(level + 1) * ctx->n, bytes, hipMemcpyDeviceToDevice, st));
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}

extern "C" cm_status cm_ntt(cm_ctx *ctx, uint64_t *dev, const int32_t *mod_idx, int32_t limbs, int32_t inverse, void *stream) {
    if (!ctx || !dev || !mod_idx || limbs < 1 || limbs > CM_NTT_MAX_LIMBS) return CM_E_INVAL;
    for (int i = 0; i < limbs; i++)
        if (mod_idx[i] < 0 || mod_idx[i] >= ctx->nmod) return CM_E_INVAL;
    // consecutive runs of modulus indices map onto the resident 0,1,2,.. table; any other list is written into the
    // context's staging array by a small kernel that carries the values as arguments (no copy, no allocation)
    bool iota = true;
    for (int i = 0; i < limbs; i++) iota &= (mod_idx[i] == mod_idx[0] + i);
    hipStream_t st = (hipStream_t)stream;
    if (iota) {
        launch_ntt(ctx, (u64 *)dev, iota_idx(ctx) + mod_idx[0], limbs, inverse != 0, st);
    } else {
        launch_set_idx(ctx->d_idx_stage, mod_idx, limbs, st);
        launch_ntt(ctx, (u64 *)dev, ctx->d_idx_stage, limbs, inverse != 0, st);
    }
    RETURN_LAUNCH_STATUS();
}

// ---- keys -------------------------------------------------------------------------------------------
extern "C" cm_status cm_keygen_secret(cm_ctx *ctx, uint64_t seed, cm_sk **out) {
    if (!ctx || !out) return CM_E_INVAL;
    CMCHK(sync_begin());
    const int n = ctx->n, h = ctx->prm.hamming;
    cm_sk *sk = new (std::nothrow) cm_sk();
    if (!sk) return CM_E_NOMEM;
    try {
    sk->noise = rng_key(seed, stream_id(ST_NOISE, 0, 0, 0));
    sk->coeffs.assign(n, 0);
    const u64 key = rng_key(seed, stream_id(ST_SECRET, 0, 0, 0));
    if (h == 0) {
        // i.i.d. uniform on {0, 1, -1}: a draw below 3*floor(2^64/3) taken mod 3
        const u64 bound = 3 * (0xFFFFFFFFFFFFFFFFULL / 3);
        static const int8_t val[3] = {0, 1, -1};
        for (int i = 0; i < n; i++) {
            u64 att = 0, v;
            do { v = rng_draw(key, (att << 32) | (u64)i); att++; } while (v >= bound);
            sk->coeffs[i] = val[v % 3];
        }
    } else {
        // h positions by a partial Fisher-Yates shuffle, one further draw bit for each sign
        std::vector<int> perm(n);
        for (int i = 0; i < n; i++) perm[i] = i;
        for (int i = 0; i < h; i++) {
            int j = i + (int)(rng_draw(key, (u64)i) % (u64)(n - i));
            std::swap(perm[i], perm[j]);
            sk->coeffs[perm[i]] = (rng_draw(key, (u64)(n + i)) & 1) ? -1 : 1;
        }
    }
    std::vector<u64> res((size_t)ctx->nmod * n);
    for (int m = 0; m < ctx->nmod; m++)
        for (int i = 0; i < n; i++) {
            int8_t c = sk->coeffs[i];
            res[(size_t)m * n + i] = c == 0 ? 0 : (c > 0 ? 1 : ctx->mod[m] - 1);
        }
    if (hipMalloc((void **)&sk->d_ntt, res.size() * 8) != hipSuccess) { delete sk; return CM_E_NOMEM; }
    if (hipMemcpy(sk->d_ntt, res.data(), res.size() * 8, hipMemcpyHostToDevice) != hipSuccess) { cm_sk_destroy(sk); return CM_E_HIP; }
    } catch (...) {
        cm_sk_destroy(sk);
        return CM_E_NOMEM;
    }
    launch_ntt(ctx, sk->d_ntt, iota_idx(ctx), ctx->nmod, false, 0);
    launch_to_mont(ctx, sk->d_ntt, iota_idx(ctx), ctx->nmod, 0);
    if (hipDeviceSynchronize() != hipSuccess) { cm_sk_destroy(sk); return CM_E_HIP; }
    *out = sk;
    return CM_OK;
}
extern "C" void cm_sk_destroy(cm_sk *sk) {
    if (!sk) return;
    hipFree(sk->d_ntt);
    delete sk;
}
extern "C" cm_status cm_sk_coeffs(const cm_ctx *ctx, const cm_sk *sk, int8_t *out) {
    if (!ctx || !sk || !out) return CM_E_INVAL;
    memcpy(out, sk->coeffs.data(), ctx->n);
    return CM_OK;
}

static cm_status make_key(cm_ctx *ctx, const cm_sk *sk, u64 g, u64 seed, EvkEntry *entry, int digits, bool stored_a) {
    const size_t n = ctx->n, nm = ctx->nmod;
    Arena A = arena_of(ctx);
    // b_j for every digit, then the generator keys of the streams of a_j; a_j itself is regenerated where it is used,
    // or, stored_a, kept behind them in multiplier form
    const size_t a_off = evk_a_offset(ctx);
    const size_t words = stored_a ? a_off + (size_t)digits * nm * n : (size_t)digits * nm * n + (size_t)digits * nm;
    if (hipMalloc((void **)&entry->d, words * 8) != hipSuccess) return CM_E_NOMEM;
    std::vector<u64> stream_keys;
    auto digs = digits_at(ctx, ctx->L);
    // P * (Q/Q_j) * ((Q/Q_j)^{-1} mod Q_j) is P on the digit's own limbs and 0 on all others: one row per digit, in the
    // spare words of the arena
    u64 *d_fac = A.misc;
    for (int j = 0; j < digits; j++) {
        u64 *b = entry->d + (size_t)j * nm * n, *a = A.tmp[1], *e = A.tmp[0];
        // a_j: drawn in the evaluation domain (no transform); limb mi uses the stream stream_id(.., j, 0) | mi
        launch_sample_uniform(ctx, a, iota_idx(ctx), (int)nm, seed, stream_id(ST_EVK_A, g, j, 0), 0);
        for (size_t mi = 0; mi < nm; mi++) stream_keys.push_back(rng_key(seed, stream_id(ST_EVK_A, g, j, 0) | (u64)mi));
        launch_sample_gauss(ctx, e, iota_idx(ctx), (int)nm, seed ^ sk->noise, stream_id(ST_EVK_E, g, j, 0), 0);
        launch_ntt(ctx, e, iota_idx(ctx), (int)nm, false, 0);
        std::vector<u64> fac(nm, 0);
        for (int i : digs[j]) {
            u64 q = ctx->mod[i], P = 1;
            for (int k = 0; k < ctx->K; k++) P = h_mulmod(P, ctx->mod[ctx->L + 1 + k] % q, q);
            fac[i] = P;
        }
        HIPCHK(hipMemcpy(d_fac, fac.data(), nm * 8, hipMemcpyHostToDevice));
        launch_evk_assemble(ctx, b, a, e, sk->d_ntt, d_fac, g, 0);
        if (stored_a) {
            u64 *dst = entry->d + a_off + (size_t)j * nm * n;
            HIPCHK(hipMemcpyAsync(dst, a, nm * n * 8, hipMemcpyDeviceToDevice, 0));
            launch_to_mont(ctx, dst, iota_idx(ctx), (int)nm, 0);
        }
        HIPCHK(hipDeviceSynchronize());
    }
    HIPCHK(hipMemcpy(entry->d + (size_t)digits * nm * n, stream_keys.data(), stream_keys.size() * 8, hipMemcpyHostToDevice));
    return CM_OK;
}

extern "C" cm_status cm_keygen_rotations(cm_ctx *ctx, const cm_sk *sk, const int32_t *steps, size_t nsteps,
                                         int32_t with_relin, uint64_t seed, cm_evk **out) {
    if (!ctx || !sk || !out || (nsteps && !steps)) return CM_E_INVAL;
    if (3 * (ctx->L + 1) < ctx->nmod) return CM_E_INVAL;
    CMCHK(sync_begin());
    cm_evk *evk = new (std::nothrow) cm_evk();
    if (!evk) return CM_E_NOMEM;
    try {
        evk->digits = (ctx->L + ctx->alpha) / ctx->alpha;
        evk->seed = seed;
        evk->stored_a = ctx->evk_stored_a;
        std::vector<u64> ids;
        for (size_t i = 0; i < nsteps; i++) ids.push_back(galois_of_step(ctx, steps[i]));
        if (with_relin) ids.push_back(0);
        for (u64 g : ids) {
            if (g == 1 || evk->keys.count(g)) continue;      // step 0 needs no key
            EvkEntry e;
            cm_status s = CM_E_NOMEM;
            try {
                s = make_key(ctx, sk, g, seed, &e, evk->digits, evk->stored_a);
                if (s == CM_OK) evk->keys[g] = e;
            } catch (...) {
                s = CM_E_NOMEM;
            }
            if (s != CM_OK) {
                hipFree(e.d);
                cm_evk_destroy(evk);
                return s;
            }
        }
    } catch (...) {
        cm_evk_destroy(evk);
        return CM_E_NOMEM;
    }
    *out = evk;
    return CM_OK;
}
extern "C" void cm_evk_destroy(cm_evk *evk) {
    if (!evk) return;
    for (auto &kv : evk->keys) hipFree(kv.second.d);
    delete evk;
}
extern "C" cm_status cm_evk_export(cm_ctx *ctx, const cm_evk *evk, int32_t step, int32_t relin, int32_t digit,
                                   int32_t comp, uint64_t *out) {
    if (!ctx || !evk || !out || digit < 0 || digit >= evk->digits || comp < 0 || comp > 1) return CM_E_INVAL;
    const u64 *key = find_key(evk, relin ? 0 : galois_of_step(ctx, step));
    if (!key) return CM_E_NOKEY;
    CMCHK(sync_begin());
    const size_t n = ctx->n, nm = ctx->nmod;
    Arena A = arena_of(ctx);
    if (comp == 0) {
        launch_from_mont(ctx, A.tmp[0], key + (size_t)digit * nm * n, iota_idx(ctx), (int)nm, 0);
    } else if (evk->stored_a) {
        launch_from_mont(ctx, A.tmp[0], key + evk_a_offset(ctx) + (size_t)digit * nm * n, iota_idx(ctx), (int)nm, 0);
    } else {
        // a_j is not stored: its limbs are the uniform streams of (seed, key id, digit), in the evaluation domain
        const u64 g = relin ? 0 : galois_of_step(ctx, step);
        launch_sample_uniform(ctx, A.tmp[0], iota_idx(ctx), (int)nm, evk->seed, stream_id(ST_EVK_A, g, digit, 0), 0);
    }
    launch_ntt(ctx, A.tmp[0], iota_idx(ctx), (int)nm, true, 0);
    HIPCHK(hipMemcpy(out, A.tmp[0], nm * n * 8, hipMemcpyDeviceToHost));
    return CM_OK;
}

// ---- plaintexts, encryption, decryption ----------------------------------------------------------------
extern "C" cm_status cm_pt_from_coeffs(cm_ctx *ctx, const int64_t *coeffs, int32_t level, double scale, cm_pt *out) {
    if (!ctx || !coeffs || !out || !out->dev || level < 0 || level > ctx->L || !(scale > 0)) return CM_E_INVAL;
    CMCHK(sync_begin());
    Arena A = arena_of(ctx);
    HIPCHK(hipMemcpy(A.misc, coeffs, (size_t)ctx->n * 8, hipMemcpyHostToDevice));
    launch_reduce_i64(ctx, out->dev, (const long long *)A.misc, iota_idx(ctx), level + 1, 0);
    launch_ntt(ctx, out->dev, iota_idx(ctx), level + 1, false, 0);
    if (out->mont) launch_to_mont(ctx, out->dev, iota_idx(ctx), level + 1, 0);
    HIPCHK(hipDeviceSynchronize());
    out->level = level;
    out->scale = scale;
    return CM_OK;
}
extern "C" cm_status cm_encode(cm_ctx *ctx, const double *re, const double *im, size_t nslots, int32_t level,
                               double scale, cm_pt *out) {
    if (!ctx || !out) return CM_E_INVAL;
    CM_TRY
    if (scale == 0) scale = ctx->prm.scale;
    std::vector<int64_t> c(ctx->n);
    CMCHK(cm_encode_coeffs(ctx, re, im, nslots, scale, c.data()));
    return cm_pt_from_coeffs(ctx, c.data(), level, scale, out);
    CM_CATCH
}

extern "C" cm_status cm_encrypt(cm_ctx *ctx, const cm_sk *sk, const cm_pt *pt, uint64_t seed, cm_ct *out) {
    if (!ctx || !sk || !pt || !pt->dev || !out || !out->dev || pt->mont) return CM_E_INVAL;
    if (pt->level < 0 || pt->level > ctx->L) return CM_E_LEVEL;
    CMCHK(sync_begin());
    const int limbs = pt->level + 1;
    const size_t n = ctx->n;
    Arena A = arena_of(ctx);
    u64 *c0 = out->dev, *c1 = out->dev + (size_t)limbs * n, *e = A.tmp[0];
    launch_sample_uniform(ctx, c1, iota_idx(ctx), limbs, seed, stream_id(ST_ENC_A, 0, 0, 0), 0);
    launch_sample_gauss(ctx, e, iota_idx(ctx), limbs, seed ^ sk->noise, stream_id(ST_ENC_E, 0, 0, 0), 0);
    launch_ntt(ctx, c1, iota_idx(ctx), limbs, false, 0);
    launch_ntt(ctx, e, iota_idx(ctx), limbs, false, 0);
    launch_encrypt(ctx, c0, c1, e, sk->d_ntt, pt->dev, limbs, 0);
    HIPCHK(hipDeviceSynchronize());
    out->level = pt->level;
    out->ncomp = 2;
    out->scale = pt->scale;
    return CM_OK;
}

extern "C" cm_status cm_decrypt(cm_ctx *ctx, const cm_sk *sk, const cm_ct *ct, cm_pt *out) {
    if (!ctx || !sk || !ct_ok(ctx, ct) || !out || !out->dev) return CM_E_INVAL;
    CMCHK(sync_begin());
    const int limbs = (ct->level >= 1 ? 1 : 0) + 1;
    launch_decrypt(ctx, out->dev, ct->dev, sk->d_ntt, ct->ncomp, ct->level + 1, limbs, 0);
    HIPCHK(hipDeviceSynchronize());
    out->level = limbs - 1;
    out->scale = ct->scale;
    out->mont = 0;
    return CM_OK;
}

extern "C" cm_status cm_decode(cm_ctx *ctx, const cm_pt *pt, double *re, double *im, size_t nslots) {
    if (!ctx || !pt || !pt->dev || !re || pt->mont || nslots > (size_t)ctx->n / 2) return CM_E_INVAL;
    if (pt->level < 0 || pt->level > 1) return CM_E_LEVEL;
    CM_TRY
    CMCHK(sync_begin());
    const size_t n = ctx->n;
    const int limbs = pt->level + 1;
    Arena A = arena_of(ctx);
    HIPCHK(hipMemcpy(A.tmp[0], pt->dev, limbs * n * 8, hipMemcpyDeviceToDevice));
    launch_ntt(ctx, A.tmp[0], iota_idx(ctx), limbs, true, 0);
    std::vector<u64> h(limbs * n);
    HIPCHK(hipMemcpy(h.data(), A.tmp[0], limbs * n * 8, hipMemcpyDeviceToHost));
    std::vector<double> m(n);
    const u64 q0 = ctx->mod[0];
    if (limbs == 1) {
        for (size_t i = 0; i < n; i++) {
            u64 x = h[i];
            m[i] = (x > q0 / 2 ? -(double)(q0 - x) : (double)x) / pt->scale;
        }
    } else {
        const u64 q1 = ctx->mod[1], inv = h_invmod(q0 % q1, q1);
        const u128 Q = (u128)q0 * q1;
        for (size_t i = 0; i < n; i++) {
            u64 x0 = h[i], x1 = h[n + i];
            u64 diff = (x1 % q1 + q1 - x0 % q1) % q1;
            u128 v = (u128)x0 + (u128)q0 * h_mulmod(diff, inv, q1);
            m[i] = (v > Q / 2 ? -(double)(Q - v) : (double)v) / pt->scale;
        }
    }
    decode_host(ctx, m, re, im, nslots);
    return CM_OK;
    CM_CATCH
}

static cm_status export_rows(cm_ctx *ctx, const u64 *dev, int ncomp, int level, bool mont, u64 *out) {
    CM_TRY
    CMCHK(sync_begin());
    const size_t n = ctx->n, rows = (size_t)ncomp * (level + 1);
    const KsLevelFull &k = ks_level_full(ctx, level);
    u64 *stage = nullptr;
    HIPCHK(hipMalloc((void **)&stage, rows * n * 8));
    if (mont)
        launch_from_mont(ctx, stage, dev, k.d_q_mods3, (int)rows, 0);
    else
        hipMemcpyAsync(stage, dev, rows * n * 8, hipMemcpyDeviceToDevice, 0);
    launch_ntt(ctx, stage, k.d_q_mods3, (int)rows, true, 0);
    hipError_t e = hipMemcpy(out, stage, rows * n * 8, hipMemcpyDeviceToHost);
    hipFree(stage);
    HIPCHK(e);
    return CM_OK;
    CM_CATCH
}
extern "C" cm_status cm_ct_export(cm_ctx *ctx, const cm_ct *ct, uint64_t *out) {
    if (!ctx || !ct_ok(ctx, ct) || !out) return CM_E_INVAL;
    return export_rows(ctx, ct->dev, ct->ncomp, ct->level, false, (u64 *)out);
}
extern "C" cm_status cm_pt_export(cm_ctx *ctx, const cm_pt *pt, uint64_t *out) {
    if (!ctx || !pt || !pt->dev || !out || pt->level < 0 || pt->level > ctx->L) return CM_E_INVAL;
    return export_rows(ctx, pt->dev, 1, pt->level, pt->mont != 0, (u64 *)out);
}

// ---- ciphertext operations ----------------------------------------------------------------------------
extern "C" cm_status cm_add(cm_ctx *ctx, const cm_ct *a, const cm_ct *b, cm_ct *out, void *stream) {
    if (!ctx || !ct_ok(ctx, a) || !ct_ok(ctx, b) || !out || !out->dev) return CM_E_INVAL;
    if (a->level != b->level || a->ncomp != b->ncomp) return CM_E_LEVEL;
    if (!same_scale(a->scale, b->scale)) return CM_E_SCALE;
    launch_add(ctx, out->dev, a->dev, b->dev, a->ncomp, a->level + 1, (hipStream_t)stream);
    out->level = a->level, out->ncomp = a->ncomp, out->scale = a->scale;
    return CM_OK;
}
extern "C" cm_status cm_mul_pt(cm_ctx *ctx, const cm_ct *a, const cm_pt *pt, cm_ct *out, void *stream) {
    if (!ctx || !ct_ok(ctx, a) || !pt || !pt->dev || !pt->mont || !out || !out->dev) return CM_E_INVAL;
    if (a->level != pt->level || a->level < 1) return CM_E_LEVEL;      // no level left to rescale into
    launch_mul_pt(ctx, out->dev, a->dev, pt->dev, a->ncomp, a->level + 1, (hipStream_t)stream);
    out->level = a->level, out->ncomp = a->ncomp, out->scale = a->scale * pt->scale;
    return CM_OK;
}
extern "C" cm_status cm_mul_ct(cm_ctx *ctx, const cm_ct *a, const cm_ct *b, cm_ct *out, void *stream) {
    if (!ctx || !ct_ok(ctx, a) || !ct_ok(ctx, b) || !out || !out->dev || a->ncomp != 2 || b->ncomp != 2) return CM_E_INVAL;
    if (a->level != b->level || a->level < 1) return CM_E_LEVEL;
    launch_tensor(ctx, out->dev, a->dev, b->dev, a->level + 1, 0, (hipStream_t)stream);
    out->level = a->level, out->ncomp = 3, out->scale = a->scale * b->scale;
    return CM_OK;
}
extern "C" cm_status cm_relinearize(cm_ctx *ctx, const cm_evk *evk, const cm_ct *a, cm_ct *out, void *stream) {
    if (!ctx || !evk || !ct_ok(ctx, a) || a->ncomp != 3 || !out || !out->dev || !evk_fits(ctx, evk)) return CM_E_INVAL;
    const u64 *key = find_key(evk, 0);
    if (!key) return CM_E_NOKEY;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    Arena A = arena_of(ctx);
    const size_t ln = (size_t)(a->level + 1) * ctx->n;
    CMCHK(ks_raise(ctx, a->dev + 2 * ln, a->level, A.digits, st));
    CMCHK(ks_apply(ctx, A.digits, key, a->level, 0, a->dev, 2, out->dev, st));
    out->level = a->level, out->ncomp = 2, out->scale = a->scale;
    return CM_OK;
    CM_CATCH
}

// the small tables a rescale reads: rows / moduli of the last limbs and of the limbs that take their residues,
// q_level^-1 mod q_i with Shoup companions, and whether the last limb's residues fit the other limbs as they are
struct RescaleTabs {
    const int *last_rows, *last_mods, *red_mods, *red_src;
    const u64 *qlinv;
    bool last_fits;
};
static cm_status rescale_core(cm_ctx *ctx, const RescaleTabs &k, const u64 *in, int ncomp, int level, u64 *out,
                              hipStream_t st, u64 *last, u64 *red, bool accumulate) {
    launch_ntt_src(ctx, last, nullptr, in, k.last_rows, k.last_mods, ncomp, true, st);
    const bool fused = ctx->n == 65536 && ncomp % 2 == 0;
    // the residues of the last limb enter the transforms of the other limbs reduced to their moduli; where the last
    // modulus is below twice the others the first pass of the fused transform takes them as they are (the transform is
    // linear and its output canonical, so the result is the same) and the reduction pass is not run
    if (!(fused && k.last_fits)) launch_rescale_reduce(ctx, red, last, ncomp, level, st);
    if (fused) {
        // the tail (in - NTT(red)) q_level^{-1} (+ out) rides on the last pass of the transform of red: the same tail as a
        // ModDown's, with `level` output rows and level+1 input rows per component and q_level^{-1} for P^{-1}
        FinishBatch fb;
        fb.items = ncomp / 2, fb.level = level - 1, fb.ext = level + 1, fb.addend_comps = 0, fb.ncomp = 2, fb.comp0 = 0;
        for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr, fb.u[r] = nullptr, fb.out[r] = nullptr, fb.g[r] = 0;
        for (int r = 0; r < fb.items; r++) {
            fb.u[r] = in + (size_t)r * 2 * (level + 1) * ctx->n, fb.out[r] = out + (size_t)r * 2 * level * ctx->n;
            fb.accum[r] = accumulate ? fb.out[r] : nullptr;
        }
        fb.pinv = k.qlinv;
        if (k.last_fits) launch_ntt_fwd_finish(ctx, red, k.red_mods, fb, st, last, k.red_src);
        else launch_ntt_fwd_finish(ctx, red, k.red_mods, fb, st);
        return CM_OK;
    }
    launch_ntt(ctx, red, k.red_mods, ncomp * level, false, st);
    launch_rescale_finish(ctx, out, in, red, k.qlinv, ncomp, level, st, accumulate);
    return CM_OK;
}
cm_status rescale_into(cm_ctx *ctx, const u64 *in, int ncomp, int level, u64 *out, hipStream_t st, u64 *last, u64 *red,
                       bool accumulate) {
    // out[comp][level][n]; must not alias in.  More than three components (several stacked
    // ciphertexts) need caller scratch: last[ncomp][n], red[ncomp][level][n].  accumulate: out += the result.
    const KsLevelFull &k = ks_level_full(ctx, level);
    Arena A = arena_of(ctx);
    if (ncomp < 1 || ncomp > RESCALE_MAX_COMPS || (ncomp > 3 && (!last || !red))) return CM_E_INVAL;
    if (!last) last = A.misc;
    if (!red) red = A.tmp[2];
    const RescaleTabs t{k.d_last_rows, k.d_last_mods, k.d_red_mods, k.d_red_src, get_qlinv(ctx, level), k.last_fits};
    return rescale_core(ctx, t, in, ncomp, level, out, st, last, red, accumulate);
}
// out[r] (+)= rescale(src_r * (pt through the Galois map g_r)) for r < cnt, src_r = mb.src[r] ([2][level+1][n]), out
// stacked at stride 2*level*n: the products are never stored; only their last limbs are formed (for the inverse
// transform), the others inside the tail of the forward transform.  Only where rescale_into would take its fused path
// and the last limb's residues fit (returns false otherwise: the caller multiplies and rescales in two steps).
bool rescale_masked_into(cm_ctx *ctx, const MulPtBatch &mb, int cnt, const u64 *pt, int level, u64 *out, hipStream_t st,
                         u64 *last, u64 *red, bool accumulate) {
    const KsLevelFull &k = ks_level_full(ctx, level);
    if (ctx->n != 65536 || !k.last_fits || cnt < 1 || cnt > CM_KS_BATCH || !last || !red) return false;
    if (ctx->two_step_masks) return false;                  // CM_OPT_TWO_STEP_MASKS: multiply, store, then rescale
    launch_mul_pt_rot_last(ctx, last, mb, cnt, pt, level + 1, st);
    launch_ntt(ctx, last, k.d_last_mods, 2 * cnt, true, st);
    FinishBatch fb;
    fb.items = cnt, fb.level = level - 1, fb.ext = level + 1, fb.addend_comps = 0, fb.ncomp = 2, fb.comp0 = 0;
    for (int r = 0; r < CM_KS_BATCH; r++) fb.addend[r] = nullptr, fb.accum[r] = nullptr, fb.u[r] = nullptr, fb.out[r] = nullptr, fb.g[r] = 0;
    for (int r = 0; r < cnt; r++) {
        fb.u[r] = mb.src[r], fb.out[r] = out + (size_t)r * 2 * level * ctx->n, fb.mul_g[r] = mb.g[r];
        fb.accum[r] = accumulate ? fb.out[r] : nullptr;
    }
    fb.mul_pt = pt;
    fb.pinv = get_qlinv(ctx, level);
    launch_ntt_fwd_finish(ctx, red, k.d_red_mods, fb, st, last, k.d_red_src);
    return true;
}
extern "C" cm_status cm_rescale(cm_ctx *ctx, const cm_ct *a, cm_ct *out, void *stream) {
    if (!ctx || !ct_ok(ctx, a) || !out || !out->dev) return CM_E_INVAL;
    if (a->level < 1) return CM_E_LEVEL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    Arena A = arena_of(ctx);
    const int level = a->level;
    u64 *dst = out->dev == a->dev ? A.tmp[1] : out->dev;
    CMCHK(rescale_into(ctx, a->dev, a->ncomp, level, dst, st));
    if (dst != out->dev)
        HIPCHK(hipMemcpyAsync(out->dev, dst, (size_t)a->ncomp * level * ctx->n * 8, hipMemcpyDeviceToDevice, st));
    out->ncomp = a->ncomp;
    out->scale = a->scale / (double)ctx->mod[level];
    out->level = level - 1;
    return CM_OK;
    CM_CATCH
}
// ---- the rescale for callers that cannot allocate -------------------------------------------------------------
// Everything cm_rescale takes from the context's arena and from per-level tables (built, hence allocated, on the first
// call at a level) lives here in one file-scope device array instead: a head of SCRATCH_HEAD words for the small
// tables of the call (written by kernels that carry the values as arguments), then the coefficient form of the last
// limbs and their residues under the other moduli.  Each GPU holds its own copy of the array at its own address; the
// address is looked up once per device and kept.  Calls on one GPU share the array: two that overlap in time race.
#define SCRATCH_HEAD 4096
#define SCRATCH_WORDS ((size_t)(4u << 20) + SCRATCH_HEAD)        // 32 MiB of limbs + the head
static __device__ __align__(256) u64 scratch[SCRATCH_WORDS];
#define SCRATCH_MAX_DEVICES 64
static u64 *g_scratch_ptr[SCRATCH_MAX_DEVICES];
// the device address of `scratch` on the current device (nullptr: the lookup failed; the error is recorded)
static u64 *scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_DEVICES) return nullptr;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) {
            cm_set_hip_error((int)e);
            return nullptr;
        }
        g_scratch_ptr[dev] = (u64 *)p;
    }
    return g_scratch_ptr[dev];
}
// called by cm_ctx_create with the context's device current
void cm_ops_device_init() { (void)scratch_of_current_device(); }

struct U64Chunk { u64 v[IDX_CHUNK_U64]; };
__global__ void k_set_u64(u64 *dst, U64Chunk c, int count) {
    const int i = threadIdx.x;
    if (i < count) dst[i] = c.v[i];
}
extern "C" cm_status cm_rescale_static(cm_ctx *ctx, const cm_ct *a, cm_ct *out, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !ct_ok(ctx, a) || !out || !out->dev || out->dev == a->dev) return CM_E_INVAL;
    if (a->level < 1) return CM_E_LEVEL;
    const int level = a->level, ncomp = a->ncomp;
    const size_t n = ctx->n;
    // head: four integer tables of at most ncomp * level entries each, then level pairs of 64-bit constants
    const size_t tab = (size_t)ncomp * level, head_words = (2 * (size_t)ncomp + 2 * tab + 1) / 2 + 2 * (size_t)level;
    if (head_words > SCRATCH_HEAD || SCRATCH_HEAD + (size_t)ncomp * n + tab * n > SCRATCH_WORDS) return CM_E_TOOBIG;
    u64 *S = scratch_of_current_device();
    if (!S) return CM_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    int h_int[2 * 3 + 2 * 3 * CM_MAX_LIMBS];
    int *h_last_rows = h_int, *h_last_mods = h_int + ncomp, *h_red_mods = h_int + 2 * ncomp, *h_red_src = h_red_mods + tab;
    bool last_fits = ctx->mod[level] < (1ULL << 52);
    for (int i = 0; i < level; i++) last_fits = last_fits && ctx->mod[level] < 2 * ctx->mod[i];
    for (int c = 0; c < ncomp; c++) {
        h_last_rows[c] = c * (level + 1) + level, h_last_mods[c] = level;
        for (int i = 0; i < level; i++) h_red_mods[c * level + i] = i, h_red_src[c * level + i] = c;
    }
    int *d_int = (int *)S;
    launch_set_idx(d_int, h_int, (int)(2 * ncomp + 2 * tab), st);
    u64 *d_qlinv = S + (2 * (size_t)ncomp + 2 * tab + 1) / 2;
    for (int base = 0; base < 2 * level; base += IDX_CHUNK_U64) {
        U64Chunk c;
        const int m = 2 * level - base < IDX_CHUNK_U64 ? 2 * level - base : IDX_CHUNK_U64;
        for (int i = 0; i < IDX_CHUNK_U64; i++) {
            c.v[i] = 0;
            if (i < m) {
                const int l = (base + i) / 2;
                const u64 q = ctx->mod[l], inv = h_invmod(ctx->mod[level] % q, q);
                c.v[i] = ((base + i) & 1) ? h_shoup(inv, q) : inv;
            }
        }
        hipLaunchKernelGGL(k_set_u64, dim3(1), dim3(IDX_CHUNK_U64), 0, st, d_qlinv + base, c, m);
    }
    u64 *last = S + SCRATCH_HEAD, *red = last + (size_t)ncomp * n;
    const RescaleTabs t{d_int, d_int + ncomp, d_int + 2 * ncomp, d_int + 2 * ncomp + tab, d_qlinv, last_fits};
    CMCHK(rescale_core(ctx, t, a->dev, ncomp, level, out->dev, st, last, red, false));
    out->ncomp = ncomp;
    out->scale = a->scale / (double)ctx->mod[level];
    out->level = level - 1;
    RETURN_LAUNCH_STATUS();
}
extern "C" cm_status cm_level_drop(cm_ctx *ctx, const cm_ct *a, int32_t level, cm_ct *out, void *stream) {
    if (!ctx || !ct_ok(ctx, a) || !out || !out->dev) return CM_E_INVAL;
    if (level < 0 || level > a->level) return CM_E_LEVEL;
    if (out->dev == a->dev && level != a->level) return CM_E_INVAL;
    const size_t n = ctx->n;
    if (out->dev != a->dev)
        for (int c = 0; c < a->ncomp; c++)
            HIPCHK(hipMemcpyAsync(out->dev + (size_t)c * (level + 1) * n, a->dev + (size_t)c * (a->level + 1) * n,
                                  (size_t)(level + 1) * n * 8, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    out->ncomp = a->ncomp, out->scale = a->scale, out->level = level;
    return CM_OK;
}

cm_status rotate_into(cm_ctx *ctx, const u64 *key, const u64 *in, int level, u64 g, u64 *out, hipStream_t st,
                      const u64 *accum, const u64 *extra) {
    // Galois map first, key switch afterwards: the map is applied while reading (the inverse NTT of
    // c1, the copy of the digits' own limbs, and the c0 added at the end), never as a pass of its own.
    // The inner product sees already mapped digits, so it runs without permutation; the ModDown
    // tail gathers c0 through the permutation.
    Arena A = arena_of(ctx);
    CMCHK(ks_raise(ctx, in + (size_t)(level + 1) * ctx->n, level, A.digits, st, g));
    const KsLevelFull &k = ks_level_full(ctx, level);
    launch_inner_product(ctx, A.u, A.u + (size_t)k.ext * ctx->n, A.digits, key, k.beta, level, 0, st, nullptr, extra);
    return moddown_into(ctx, A.u, level, in, 1, g, out, accum, st);
}
extern "C" cm_status cm_rotate(cm_ctx *ctx, const cm_evk *evk, const cm_ct *in, int32_t step, cm_ct *out, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !ct_ok(ctx, in) || in->ncomp != 2 || !out || !out->dev || !evk_fits(ctx, evk)) return CM_E_INVAL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    const u64 g = galois_of_step(ctx, step);
    if (g == 1) {
        if (out->dev != in->dev)
            HIPCHK(hipMemcpyAsync(out->dev, in->dev, cm_ct_words(ctx, in->level, 2) * 8, hipMemcpyDeviceToDevice, st));
    } else {
        const u64 *key = find_key(evk, g);
        if (!key) return CM_E_NOKEY;
        if (out->dev == in->dev) {      // the last kernel gathers from `in`: go through a temporary
            Arena A = arena_of(ctx);
            CMCHK(rotate_into(ctx, key, in->dev, in->level, g, A.tmp[0], st));
            HIPCHK(hipMemcpyAsync(out->dev, A.tmp[0], cm_ct_words(ctx, in->level, 2) * 8, hipMemcpyDeviceToDevice, st));
        } else {
            CMCHK(rotate_into(ctx, key, in->dev, in->level, g, out->dev, st));
        }
    }
    out->level = in->level, out->ncomp = 2, out->scale = in->scale;
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
extern "C" cm_status cm_rotate_hoisted(cm_ctx *ctx, const cm_evk *evk, const cm_ct *in, const int32_t *steps,
                                       size_t nsteps, cm_ct *outs, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !ct_ok(ctx, in) || in->ncomp != 2 || !steps || !outs || !evk_fits(ctx, evk)) return CM_E_INVAL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    for (size_t i = 0; i < nsteps; i++) {
        if (!outs[i].dev || outs[i].dev == in->dev) return CM_E_INVAL;
        u64 g = galois_of_step(ctx, steps[i]);
        if (g != 1 && !find_key(evk, g)) return CM_E_NOKEY;
    }
    Arena A = arena_of(ctx);
    const size_t ln = (size_t)(in->level + 1) * ctx->n;
    CMCHK(ks_raise(ctx, in->dev + ln, in->level, A.digits, st));
    std::vector<const u64 *> keys;
    std::vector<u64> gs;
    std::vector<u64 *> dst;
    for (size_t i = 0; i < nsteps; i++) {
        u64 g = galois_of_step(ctx, steps[i]);
        if (g == 1) {
            HIPCHK(hipMemcpyAsync(outs[i].dev, in->dev, 2 * ln * 8, hipMemcpyDeviceToDevice, st));
        } else {
            keys.push_back(find_key(evk, g)), gs.push_back(g), dst.push_back(outs[i].dev);
        }
        outs[i].level = in->level, outs[i].ncomp = 2, outs[i].scale = in->scale;
    }
    CMCHK(ks_apply_many(ctx, A.digits, in->level, (int)keys.size(), keys.data(), gs.data(), in->dev, dst.data(), st));
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
