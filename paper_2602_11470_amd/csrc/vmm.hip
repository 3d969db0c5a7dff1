// Packed homomorphic vector-matrix product (Sec. 4.1, App. C / Algorithm 1): plan building
// (slot layout, weight diagonals, rotation amounts) and the device driver.
//
// Slots are written i = b*t + r (block b, residue r), t = S/d for the shorter vector length d,
// t' = S/(alpha d) for the longer one.  Rotation amounts of the printed algorithm are read in
// slots as: preprocess 2^i (t-1); baby step j t' t; giant step r_i t' t; reduce 2^l; and
// r_o = d/(t' r_i), the choice for which r_i r_o t' = d.
//
// Token-batched plans (the prompt phase, Sec. 5.4): residue tau of block b holds element b of
// token tau, so nothing is replicated before and nothing summed after; the product is the
// diagonal method over all d diagonals, every rotation a whole number of blocks (baby step j t,
// giant step r_i t), every weight diagonal repeated over the residues.
#include <math.h>

#include <thread>
#include <utility>

#include "kernels.h"

struct cm_vmm_plan {
    cm_ctx *ctx = nullptr;
    int S, d, alpha, t, tp, t1, t2, r_i, r_o, M, tau, d_in, d_out, level;
    bool expand, contract;
    bool tokens = false;       // token-batched: t tokens per ciphertext, square shapes only
    double pt_scale;
    std::vector<int> pre_steps, baby_steps, reduce_steps;
    int giant_step;
    bool raised = false;       // sums of the baby steps stay in the extended basis (one ModDown per giant step)
    bool direct = false;       // giant steps unrolled: independent rotations by k*giant_step, one shared ModDown
    bool unrolled = false;     // the two rotate-and-add ladders unrolled too; the whole product in the extended basis
    std::vector<std::vector<int>> pre_groups, reduce_groups;   // rotation amounts of each run of <= 3 ladder steps
    KsManyTables many;         // direct: tables for raising the r_o - 1 inner sums at once
    u64 *d_many = nullptr;     // direct: r_o - 1 ciphertexts, their coefficient-domain c1 and their raised digits
    int pt_limbs;              // level+1, or level+1+K when raised
    int *d_pt_mods = nullptr;  // modulus index of every plaintext limb
    u64 *d_pts = nullptr;      // r_i*r_o plaintexts of pt_limbs limbs, multiplier form, blocked by 64 coefficients
    u64 *d_work = nullptr;     // r_i baby + r_o inner ciphertexts of 2*pt_limbs limbs, 3 temporary ciphertexts, one more sum
};

static int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) l++;
    return l;
}
static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

static cm_status plan_shape(cm_ctx *ctx, int d_in, int d_out, int r_i, int tau, int level, double pt_scale,
                            bool tokens, bool cheap_babies, cm_vmm_plan *p) {
    if (d_in < 1 || d_out < 1 || level < 1 || level > ctx->L) return level < 1 ? CM_E_LEVEL : CM_E_INVAL;
    p->ctx = ctx;
    p->S = ctx->n / 2;
    p->d_in = d_in, p->d_out = d_out;
    p->d = d_in < d_out ? d_in : d_out;
    int big = d_in < d_out ? d_out : d_in;
    if (!pow2(p->d) || !pow2(big) || big > p->S) return CM_E_LAYOUT;
    p->alpha = big / p->d;
    p->expand = d_out > d_in, p->contract = d_in > d_out;
    p->t = p->S / p->d, p->tp = p->S / big;
    p->t1 = p->contract ? p->tp : p->t;
    p->t2 = p->contract ? p->t : p->tp;
    p->tokens = tokens;
    if (tokens) {
        if (d_in != d_out) return CM_E_LAYOUT;
        p->tp = p->t1 = p->t2 = 1;          // rotations count blocks of t; no preprocess, no reduce
    }
    p->M = p->d / p->tp;
    if (p->M < 1) return CM_E_LAYOUT;
    if (r_i == 0) {
        r_i = 1 << ((ilog2(p->M) + 1) / 2);
        // twice that where the baby steps stay in the extended basis (one inner product each, no ModUp or ModDown of
        // their own): they are then several times cheaper than the giant steps, each of which raises a ciphertext
        if (cheap_babies && 2 * r_i <= p->M) r_i *= 2;
    }
    if (!pow2(r_i) || p->M % r_i) return CM_E_LAYOUT;
    p->r_i = r_i, p->r_o = p->M / r_i;
    if (tau < 0 || tau >= p->t2) return CM_E_LAYOUT;
    p->tau = tau, p->level = level;
    p->pt_scale = pt_scale > 0 ? pt_scale : ctx->prm.scale;
    for (int i = 0; i < ilog2(p->t1); i++) p->pre_steps.push_back((1 << i) * (p->t - 1));
    for (int j = 0; j < r_i; j++) p->baby_steps.push_back(j * p->tp * p->t);
    p->giant_step = r_i * p->tp * p->t;
    // block of t2 slots sums into residue tau: rotate right where the bit of tau is set
    for (int l = 0; l < ilog2(p->t2); l++) p->reduce_steps.push_back(((tau >> l) & 1) ? -(1 << l) : (1 << l));
    return CM_OK;
}

static int in_slot(const cm_vmm_plan *p, int a) {
    return p->contract ? (a % p->d) * p->t + (a / p->d) * p->tp : a * p->t;
}

// Input index present in every slot after the preprocess step, found by moving index labels
// through the same rotate-and-add steps.
static std::vector<int> source_labels(const cm_vmm_plan *p) {
    const int S = p->S;
    std::vector<int> lab(S, -1), nxt(S);
    if (p->tokens) {
        for (int i = 0; i < S; i++) lab[i] = i / p->t;
        return lab;
    }
    for (int a = 0; a < p->d_in; a++) lab[in_slot(p, a)] = a;
    for (int r : p->pre_steps) {
        for (int i = 0; i < S; i++) {
            int from = lab[(i + r) % S];            // Rot(c, r)[i] = c[i + r]
            nxt[i] = from >= 0 ? from : lab[i];
        }
        lab.swap(nxt);
    }
    return lab;
}

// Slot vector of weight plaintext (j, k): the product at slot i of baby rotation j ends, after k
// giant rotations and the reduce step, in the block of t2 slots that owns one output index.
static void diag_slots(const cm_vmm_plan *p, const std::vector<int> &lab, const double *W, int j, int k,
                       std::vector<double> &out) {
    const int S = p->S;
    out.resize(S);
    for (int i = 0; i < S; i++) {
        int row = lab[(i + p->baby_steps[j]) % S];
        int blk = (int)((((long long)i - (long long)k * p->giant_step) % S + S) % S) / (p->tokens ? p->t : p->t2);
        int col = p->expand ? blk / p->alpha + (blk % p->alpha) * p->d : blk;
        out[i] = W[(size_t)row * p->d_out + col];
    }
}

// A ladder c <- c + Rot(c, s_l) over a run of steps equals c + the rotations of c by every non-empty
// subset sum of the run.  The ladder is cut into ceil(L/3) runs of as equal length as possible, the
// longer ones first (at most seven rotations of one ciphertext per run).
static std::vector<std::vector<int>> ladder_groups(const std::vector<int> &steps) {
    std::vector<std::vector<int>> out;
    const size_t L = steps.size(), runs = (L + 2) / 3;
    size_t i = 0;
    for (size_t r = 0; r < runs; r++) {
        const size_t g = L / runs + (r < L % runs ? 1 : 0);
        std::vector<int> amounts;
        for (unsigned b = 1; b < (1u << g); b++) {
            int a = 0;
            for (size_t l = 0; l < g; l++)
                if ((b >> l) & 1) a += steps[i + l];
            amounts.push_back(a);
        }
        i += g;
        out.push_back(amounts);
    }
    return out;
}

static cm_status plan_alloc(cm_vmm_plan *p, bool raised, bool direct, bool unrolled) {
    cm_ctx *ctx = p->ctx;
    p->raised = raised, p->direct = direct, p->unrolled = unrolled;
    if (unrolled) p->pre_groups = ladder_groups(p->pre_steps), p->reduce_groups = ladder_groups(p->reduce_steps);
    p->pt_limbs = p->level + 1 + (raised ? ctx->K : 0);
    std::vector<int> mods;
    for (int i = 0; i <= p->level; i++) mods.push_back(i);
    for (int k = 0; raised && k < ctx->K; k++) mods.push_back(ctx->L + 1 + k);
    const size_t n = ctx->n, ptw = (size_t)p->pt_limbs * n, ctw = 2 * (size_t)(p->level + 1) * n;
    if (hipMalloc((void **)&p->d_pt_mods, mods.size() * sizeof(int)) != hipSuccess) return CM_E_NOMEM;
    if (hipMemcpy(p->d_pt_mods, mods.data(), mods.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess) return CM_E_HIP;
    if (hipMalloc((void **)&p->d_pts, (size_t)p->M * ptw * 8) != hipSuccess) return CM_E_NOMEM;
    // r_i baby + r_o inner ciphertexts, 3 temporaries on the ciphertext limbs, one more on the plaintext limbs
    if (hipMalloc((void **)&p->d_work, ((size_t)(p->r_i + p->r_o + 1) * 2 * ptw + 3 * ctw) * 8) != hipSuccess) return CM_E_NOMEM;
    if (direct && p->r_o > 1) {
        const KsLevel &k = ks_level(ctx, p->level);
        const size_t cnt = p->r_o - 1, per = ctw + (size_t)(p->level + 1) * n + (size_t)k.beta * k.ext * n;
        cm_status s = ks_many_tables_create(ctx, p->level, (int)cnt, &p->many);
        if (s != CM_OK) return s;
        if (hipMalloc((void **)&p->d_many, cnt * per * 8) != hipSuccess) return CM_E_NOMEM;
    }
    return CM_OK;
}

// plaintext polynomial of integer coefficients on the plan's limbs, evaluation domain, multiplier form
static cm_status plan_load_diag(cm_vmm_plan *p, int idx, const int64_t *coeffs) {
    cm_ctx *ctx = p->ctx;
    u64 *stage = p->d_work, *plain = stage + ctx->n;          // the work area is free until the first product
    HIPCHK(hipMemcpy(stage, coeffs, (size_t)ctx->n * 8, hipMemcpyHostToDevice));
    launch_reduce_i64(ctx, plain, (const long long *)stage, p->d_pt_mods, p->pt_limbs, 0);
    launch_ntt_rows(ctx, plain, nullptr, p->d_pt_mods, p->pt_limbs, false, 0);
    launch_to_mont(ctx, plain, p->d_pt_mods, p->pt_limbs, 0);
    launch_pt_block(ctx, p->d_pts, plain, p->pt_limbs, p->r_i, p->r_o, idx / p->r_o, idx % p->r_o, true, 0);
    HIPCHK(hipDeviceSynchronize());
    return CM_OK;
}

extern "C" cm_status cm_vmm_plan_create_ex(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i, int32_t tau,
                                           int32_t level, double pt_scale, const double *W, const int64_t *coeffs,
                                           uint32_t flags, cm_vmm_plan **out) {
    if (!ctx || (!W == !coeffs) || !out ||
        (flags & ~(uint32_t)(CM_VMM_RAISED_SUMS | CM_VMM_DIRECT_GIANTS | CM_VMM_TOKEN_BATCH | CM_VMM_UNROLLED_LADDERS)))
        return CM_E_INVAL;
    const bool unrolled = (flags & CM_VMM_UNROLLED_LADDERS) != 0;
    const bool direct = unrolled || (flags & CM_VMM_DIRECT_GIANTS) != 0, raised = direct || (flags & CM_VMM_RAISED_SUMS) != 0;
    cm_vmm_plan *p = new (std::nothrow) cm_vmm_plan();
    if (!p) return CM_E_NOMEM;
    try {
    cm_status s = plan_shape(ctx, d_in, d_out, r_i, tau, level, pt_scale, (flags & CM_VMM_TOKEN_BATCH) != 0,
                             raised || (flags & CM_VMM_TOKEN_BATCH) != 0, p);
    if (s == CM_OK) s = plan_alloc(p, raised, direct, unrolled);
    if (s != CM_OK) { cm_vmm_plan_destroy(p); return s; }
    if (coeffs) {
        for (int idx = 0; idx < p->M && s == CM_OK; idx++) s = plan_load_diag(p, idx, coeffs + (size_t)idx * ctx->n);
        if (s != CM_OK) { cm_vmm_plan_destroy(p); return s; }
        *out = p;
        return CM_OK;
    }
    const std::vector<int> lab = source_labels(p);
    const int n = ctx->n, batch = 16;
    std::vector<std::vector<int64_t>> cf(batch, std::vector<int64_t>(n));
    std::vector<cm_status> st(batch);
    for (int base = 0; base < p->M && s == CM_OK; base += batch) {
        int cnt = p->M - base < batch ? p->M - base : batch;
        std::vector<std::thread> th;
        for (int b = 0; b < cnt; b++)
            th.emplace_back([&, b]() {
                int idx = base + b, j = idx / p->r_o, k = idx % p->r_o;
                std::vector<double> slots;
                diag_slots(p, lab, W, j, k, slots);
                st[b] = cm_encode_coeffs(ctx, slots.data(), nullptr, slots.size(), p->pt_scale, cf[b].data());
            });
        for (auto &t : th) t.join();
        for (int b = 0; b < cnt && s == CM_OK; b++) {
            s = st[b];
            if (s == CM_OK) s = plan_load_diag(p, base + b, cf[b].data());
        }
    }
    if (s != CM_OK) { cm_vmm_plan_destroy(p); return s; }
    *out = p;
    return CM_OK;
    } catch (...) {                  // host allocation (tables, encoder threads): the plan's device memory is released
        cm_vmm_plan_destroy(p);
        return CM_E_NOMEM;
    }
}
extern "C" cm_status cm_vmm_plan_create(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i, int32_t tau,
                                        int32_t level, double pt_scale, const double *W, cm_vmm_plan **out) {
    if (!W) return CM_E_INVAL;
    return cm_vmm_plan_create_ex(ctx, d_in, d_out, r_i, tau, level, pt_scale, W, nullptr, 0, out);
}
extern "C" cm_status cm_vmm_plan_create_from_coeffs(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i,
                                                    int32_t tau, int32_t level, double pt_scale,
                                                    const int64_t *coeffs, cm_vmm_plan **out) {
    if (!coeffs) return CM_E_INVAL;
    return cm_vmm_plan_create_ex(ctx, d_in, d_out, r_i, tau, level, pt_scale, nullptr, coeffs, 0, out);
}

extern "C" void cm_vmm_plan_destroy(cm_vmm_plan *plan) {
    if (!plan) return;
    ks_many_tables_destroy(&plan->many);
    hipFree(plan->d_many);
    hipFree(plan->d_pt_mods);
    hipFree(plan->d_pts);
    hipFree(plan->d_work);
    delete plan;
}

static std::vector<int> plan_all_steps(const cm_vmm_plan *p) {
    std::vector<int> all;
    if (p->unrolled) for (const auto &g : p->pre_groups) all.insert(all.end(), g.begin(), g.end());
    else all = p->pre_steps;
    for (int j = 1; j < p->r_i; j++) all.push_back(p->baby_steps[j]);
    for (int k = 1; k < p->r_o; k++)
        if (k == 1 || p->direct) all.push_back(k * p->giant_step);
    if (p->unrolled) for (const auto &g : p->reduce_groups) all.insert(all.end(), g.begin(), g.end());
    else all.insert(all.end(), p->reduce_steps.begin(), p->reduce_steps.end());
    return all;
}
extern "C" int32_t cm_vmm_plan_steps(const cm_vmm_plan *p, int32_t *steps, int32_t cap) {
    if (!p) return 0;
    try {
        std::vector<int> all = plan_all_steps(p);
        for (int i = 0; i < (int)all.size() && i < cap && steps; i++) steps[i] = all[i];
        return (int32_t)all.size();
    } catch (...) {
        return 0;
    }
}
extern "C" cm_status cm_vmm_plan_info(const cm_vmm_plan *p, int32_t *r_i, int32_t *r_o, int32_t *n_rot) {
    if (!p) return CM_E_INVAL;
    if (r_i) *r_i = p->r_i;
    if (r_o) *r_o = p->r_o;
    if (n_rot) {
        size_t ladders = p->pre_steps.size() + p->reduce_steps.size();
        if (p->unrolled) {
            ladders = 0;
            for (const auto &g : p->pre_groups) ladders += g.size();
            for (const auto &g : p->reduce_groups) ladders += g.size();
        }
        *n_rot = (int)ladders + (p->r_i - 1) + (p->r_o - 1);
    }
    return CM_OK;
}
extern "C" cm_status cm_vmm_plan_diag_export(cm_ctx *ctx, const cm_vmm_plan *p, int32_t j, int32_t k, uint64_t *out) {
    if (!ctx || !p || !out || j < 0 || j >= p->r_i || k < 0 || k >= p->r_o) return CM_E_INVAL;
    const size_t words = (size_t)p->pt_limbs * ctx->n;
    u64 *tmp = nullptr;
    HIPCHK(hipDeviceSynchronize());
    if (hipMalloc((void **)&tmp, words * 8) != hipSuccess) return CM_E_NOMEM;
    launch_pt_block(ctx, p->d_pts, tmp, p->pt_limbs, p->r_i, p->r_o, j, k, false, 0);
    launch_from_mont(ctx, tmp, tmp, p->d_pt_mods, p->pt_limbs, 0);
    launch_ntt_rows(ctx, tmp, nullptr, p->d_pt_mods, p->pt_limbs, true, 0);
    hipError_t e = hipMemcpy(out, tmp, words * 8, hipMemcpyDeviceToHost);
    hipFree(tmp);
    return e == hipSuccess ? CM_OK : CM_E_HIP;
}

// The same product with the sums of the baby steps kept in the extended basis: hoisted rotations stop
// before their ModDown (u + P sigma(c0), u1), the plaintext products are summed on level+1+K limbs,
// and every inner_k is divided by P inside the giant step that consumes it.
// First half: preprocess and baby steps of x into the plan's own work area (babies[r_i][2][ext][n]).
static cm_status vmm_raised_babies(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *p, const cm_ct *x, hipStream_t st) {
    const int level = p->level, limbs = level + 1, ext = p->pt_limbs;
    const size_t n = ctx->n, ctw = 2 * (size_t)limbs * n, ptw = (size_t)limbs * n, rw = 2 * (size_t)ext * n;
    auto key_of = [&](int step) { return find_key(evk, galois_of_step(ctx, step)); };
    u64 *babies = p->d_work, *inner = babies + (size_t)p->r_i * rw, *t0 = inner + (size_t)p->r_o * rw;
    u64 *t1 = t0 + ctw;
    if (p->unrolled) {
        // The whole product stays in the extended basis.  R = (P c0, P c1); every run of the preprocess ladder adds
        // the hoisted rotations of R by its subset sums (one raise of ModDown(R1), one launch summing all of them
        // with sigma(R0) and R itself), between two buffers so that the last run ends in baby slot 0.
        u64 *spare = t0 + 3 * ctw;
        const size_t ngroups = p->pre_groups.size();
        u64 *cur = (ngroups & 1) ? spare : babies, *nxt = (ngroups & 1) ? babies : spare;
        launch_raise_by_P(ctx, cur, x->dev, level, st);
        const KsLevel &kl = ks_level(ctx, level);
        for (size_t gi = 0; gi < ngroups; gi++) {
            const u64 *c1 = x->dev + ptw;                     // ModDown(P c1) = c1 exactly
            if (gi) {
                CMCHK(moddown_second_keep(ctx, cur, level, t0, st));
                c1 = t0 + ptw;
            }
            u64 *digits = arena_digits(ctx);
            CMCHK(ks_raise(ctx, c1, level, digits, st));
            IpBatch b;
            b.nz = 1, b.nsum = (int)p->pre_groups[gi].size();
            for (int s = 0; s < b.nsum; s++) {
                const int a = p->pre_groups[gi][s];
                b.it[s].dig = digits, b.it[s].key = key_of(a), b.it[s].c0 = cur, b.it[s].c0_ext = 1;
                b.it[s].g = (unsigned)galois_of_step(ctx, a);
            }
            b.out[0] = nxt, b.extra[0] = cur;
            launch_inner_product_batch(ctx, b, kl.beta, level, st);
            std::swap(cur, nxt);
        }
        if (p->r_i > 1) {
            const u64 *c1 = x->dev + ptw;
            if (ngroups) {
                CMCHK(moddown_second_keep(ctx, babies, level, t0, st));
                c1 = t0 + ptw;
            }
            u64 *digits = arena_digits(ctx);
            CMCHK(ks_raise(ctx, c1, level, digits, st));
            std::vector<const u64 *> keys;
            std::vector<u64> gs;
            std::vector<u64 *> dst;
            for (int j = 1; j < p->r_i; j++) {
                keys.push_back(key_of(p->baby_steps[j]));
                gs.push_back(galois_of_step(ctx, p->baby_steps[j]));
                dst.push_back(babies + (size_t)j * rw);
            }
            CMCHK(ks_apply_many_raised(ctx, digits, level, p->r_i - 1, keys.data(), gs.data(), babies, dst.data(), st, true));
        }
        return CM_OK;
    }
    // 1. preprocess (rotate-and-add between two buffers)
    u64 *c = t0, *other = t1;
    HIPCHK(hipMemcpyAsync(c, x->dev, ctw * 8, hipMemcpyDeviceToDevice, st));
    for (int r : p->pre_steps) {
        CMCHK(rotate_into(ctx, key_of(r), c, level, galois_of_step(ctx, r), other, st, c));
        std::swap(c, other);
    }
    // 2. baby steps, left in the extended basis
    launch_raise_by_P(ctx, babies, c, level, st);
    if (p->r_i > 1) {
        u64 *digits = arena_digits(ctx);
        CMCHK(ks_raise(ctx, c + ptw, level, digits, st));
        std::vector<const u64 *> keys;
        std::vector<u64> gs;
        std::vector<u64 *> dst;
        for (int j = 1; j < p->r_i; j++) {
            keys.push_back(key_of(p->baby_steps[j]));
            gs.push_back(galois_of_step(ctx, p->baby_steps[j]));
            dst.push_back(babies + (size_t)j * rw);
        }
        CMCHK(ks_apply_many_raised(ctx, digits, level, p->r_i - 1, keys.data(), gs.data(), c, dst.data(), st));
    }
    return CM_OK;
}
// Second half: products with the plan's own weights against the given baby ciphertexts (its own, or
// those of another plan of the same shape that saw the same input), giant steps, reduce, rescale.
static cm_status vmm_raised_finish(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *p, const u64 *babies, const cm_ct *x,
                                   cm_ct *y, hipStream_t st) {
    const int level = p->level, limbs = level + 1, ext = p->pt_limbs;
    const size_t n = ctx->n, ctw = 2 * (size_t)limbs * n, rw = 2 * (size_t)ext * n;
    auto key_of = [&](int step) { return find_key(evk, galois_of_step(ctx, step)); };
    u64 *inner = p->d_work + (size_t)p->r_i * rw, *t0 = inner + (size_t)p->r_o * rw;
    u64 *t1 = t0 + ctw, *t2 = t1 + ctw;
    const int r_o = p->r_o;
    launch_vmm_mac(ctx, inner, babies, p->d_pts, p->r_i, r_o, ext, level, rw, 0, r_o, st);
    u64 *acc = t1, *other = t2;
    if (p->direct) {
        // giant steps unrolled: the second component of inner_k is divided by P and raised digit by digit
        // (all k at once); its first component is never divided: it goes through the Galois map on all
        // limbs of the extended basis and joins the sum as it is.  Every rotation by k*G stays in the
        // extended basis and joins inner_0; one ModDown for the whole sum.
        const KsLevel &kl = ks_level(ctx, level);
        const int cnt = r_o - 1;
        u64 *cts = p->d_many, *ksin = cts + (size_t)cnt * ctw, *digs = ksin + (size_t)cnt * limbs * n;
        std::vector<u64 *> outs;
        for (int k = 0; k < cnt; k++) outs.push_back(cts + (size_t)k * ctw);
        CMCHK(moddown_many_second(ctx, inner + rw, level, cnt, outs.data(), st));
        CMCHK(ks_raise_many(ctx, p->many, cts, ksin, digs, st));
        for (int k0 = 1; k0 < r_o; k0 += IP_MAX_ITEMS) {          // all rotations summed onto inner_0 by one launch
            IpBatch b;
            b.nz = 1, b.nsum = r_o - k0 < IP_MAX_ITEMS ? r_o - k0 : IP_MAX_ITEMS;
            for (int s = 0; s < b.nsum; s++) {
                const int k = k0 + s;
                b.it[s].dig = digs + (size_t)(k - 1) * kl.beta * kl.ext * n, b.it[s].key = key_of(k * p->giant_step);
                b.it[s].c0 = inner + (size_t)k * rw, b.it[s].c0_ext = 1;
                b.it[s].g = (unsigned)galois_of_step(ctx, k * p->giant_step);
            }
            b.out[0] = inner, b.extra[0] = inner;
            launch_inner_product_batch(ctx, b, kl.beta, level, st);
        }
        u64 *total = inner;
        if (p->unrolled) {
            // the reduce ladder, run by run, still in the extended basis (between inner_0 and the spare buffer)
            u64 *spare = t0 + 3 * ctw, *nxt = spare;
            for (const auto &grp : p->reduce_groups) {
                CMCHK(moddown_second_keep(ctx, total, level, t0, st));
                u64 *digits = arena_digits(ctx);
                CMCHK(ks_raise(ctx, t0 + (size_t)limbs * n, level, digits, st));
                IpBatch b;
                b.nz = 1, b.nsum = (int)grp.size();
                for (int s = 0; s < b.nsum; s++) {
                    b.it[s].dig = digits, b.it[s].key = key_of(grp[s]), b.it[s].c0 = total, b.it[s].c0_ext = 1;
                    b.it[s].g = (unsigned)galois_of_step(ctx, grp[s]);
                }
                b.out[0] = nxt, b.extra[0] = total;
                launch_inner_product_batch(ctx, b, kl.beta, level, st);
                std::swap(total, nxt);
            }
        }
        CMCHK(moddown_into(ctx, total, level, nullptr, 0, 0, acc, nullptr, st));
    } else {
        // giant steps, Horner form: acc <- Rot(acc) + ModDown-ed inner_k in one key switch
        CMCHK(moddown_into(ctx, inner + (size_t)(r_o - 1) * rw, level, nullptr, 0, 0, acc, nullptr, st));
        for (int k = r_o - 2; k >= 0; k--) {
            CMCHK(rotate_into(ctx, key_of(p->giant_step), acc, level, galois_of_step(ctx, p->giant_step), other, st,
                              nullptr, inner + (size_t)k * rw));
            std::swap(acc, other);
        }
    }
    // 3. reduce inside the ciphertext
    for (int r : p->reduce_steps) {
        if (p->unrolled) break;                               // done above, before the ModDown
        CMCHK(rotate_into(ctx, key_of(r), acc, level, galois_of_step(ctx, r), other, st, acc));
        std::swap(acc, other);
    }
    CMCHK(rescale_into(ctx, acc, 2, level, y->dev, st));
    y->level = level - 1, y->ncomp = 2;
    y->scale = x->scale * p->pt_scale / (double)ctx->mod[level];
    RETURN_LAUNCH_STATUS();
}
static cm_status vmm_pt_raised(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *p, const cm_ct *x, cm_ct *y,
                               hipStream_t st) {
    CMCHK(vmm_raised_babies(ctx, evk, p, x, st));
    return vmm_raised_finish(ctx, evk, p, p->d_work, x, y, st);
}

static cm_status plan_keys_present(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *p) {
    auto key_of = [&](int step) { return find_key(evk, galois_of_step(ctx, step)); };
    for (int r : plan_all_steps(p)) if (!key_of(r)) return CM_E_NOKEY;
    return CM_OK;
}

extern "C" cm_status cm_vmm_pt_multi(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *const *plans, int32_t nplans,
                                     const cm_ct *x, cm_ct *const *ys, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !plans || nplans < 1 || !x || !x->dev || x->ncomp != 2 || !ys || !evk_fits(ctx, evk)) return CM_E_INVAL;
    CM_TRY
    const cm_vmm_plan *p0 = plans[0];
    for (int i = 0; i < nplans; i++) {
        const cm_vmm_plan *p = plans[i];
        if (!p || p->ctx != ctx || !ys[i] || !ys[i]->dev || !p->raised) return CM_E_INVAL;
        if (p->level != p0->level || p->d_in != p0->d_in || p->d_out != p0->d_out || p->r_i != p0->r_i ||
            p->tokens != p0->tokens || p->unrolled != p0->unrolled)
            return CM_E_LAYOUT;
        for (int j = 0; j < i; j++)
            if (plans[j] == p) return CM_E_INVAL;         // a plan's work area holds one product at a time
        cm_status s = plan_keys_present(ctx, evk, p);
        if (s != CM_OK) return s;
    }
    if (x->level != p0->level) return CM_E_LEVEL;
    hipStream_t st = (hipStream_t)stream;
    CMCHK(vmm_raised_babies(ctx, evk, p0, x, st));
    for (int i = 0; i < nplans; i++) CMCHK(vmm_raised_finish(ctx, evk, plans[i], p0->d_work, x, ys[i], st));
    return CM_OK;
    CM_CATCH
}

extern "C" cm_status cm_vmm_pt(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *p, const cm_ct *x, cm_ct *y,
                               void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !p || !x || !x->dev || !y || !y->dev || x->ncomp != 2 || p->ctx != ctx || !evk_fits(ctx, evk)) return CM_E_INVAL;
    if (x->level != p->level) return CM_E_LEVEL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    const int level = p->level, limbs = level + 1;
    const size_t n = ctx->n, ctw = 2 * (size_t)limbs * n, ptw = (size_t)limbs * n;
    // every key must be there before anything is enqueued
    CMCHK(plan_keys_present(ctx, evk, p));
    auto key_of = [&](int step) { return find_key(evk, galois_of_step(ctx, step)); };
    if (p->raised) return vmm_pt_raised(ctx, evk, p, x, y, st);
    u64 *babies = p->d_work, *inner = babies + (size_t)p->r_i * ctw, *tmp = inner + (size_t)p->r_o * ctw;
    // 1. preprocess: c <- c + Rot(c, 2^i (t-1)).  A rotate-and-add writes to the other of two buffers
    //    (its last kernel gathers c0 of its input through the permutation, so it cannot run in
    //    place); start in the one that leaves the result in baby slot 0.
    u64 *c = (p->pre_steps.size() & 1) ? tmp : babies, *other = (p->pre_steps.size() & 1) ? babies : tmp;
    HIPCHK(hipMemcpyAsync(c, x->dev, ctw * 8, hipMemcpyDeviceToDevice, st));
    for (int r : p->pre_steps) {
        CMCHK(rotate_into(ctx, key_of(r), c, level, galois_of_step(ctx, r), other, st, c));
        std::swap(c, other);
    }
    // 2. baby steps: rotations of the same ciphertext share its raised digits
    if (p->r_i > 1) {
        u64 *digits = arena_digits(ctx);
        CMCHK(ks_raise(ctx, c + ptw, level, digits, st));
        std::vector<const u64 *> keys;
        std::vector<u64> gs;
        std::vector<u64 *> dst;
        for (int j = 1; j < p->r_i; j++) {
            keys.push_back(key_of(p->baby_steps[j]));
            gs.push_back(galois_of_step(ctx, p->baby_steps[j]));
            dst.push_back(babies + (size_t)j * ctw);
        }
        CMCHK(ks_apply_many(ctx, digits, level, p->r_i - 1, keys.data(), gs.data(), c, dst.data(), st));
    }
    //    multiply-accumulate: inner_k = sum_j baby_j * p_{j,k}; streams every weight plaintext once
    const int r_o = p->r_o;
    launch_vmm_mac(ctx, inner, babies, p->d_pts, p->r_i, r_o, limbs, level, ctw, 0, r_o, st);
    //    giant steps, Horner form
    u64 *acc = inner + (size_t)(r_o - 1) * ctw;
    for (int k = r_o - 2; k >= 0; k--) {
        u64 *nxt = inner + (size_t)k * ctw;                  // inner_k + Rot(acc), written over inner_k
        CMCHK(rotate_into(ctx, key_of(p->giant_step), acc, level, galois_of_step(ctx, p->giant_step), nxt, st, nxt));
        acc = nxt;
    }
    // 3. reduce inside the ciphertext (two buffers again; baby slot 0 is free by now)
    other = acc == babies ? tmp : babies;
    for (int r : p->reduce_steps) {
        CMCHK(rotate_into(ctx, key_of(r), acc, level, galois_of_step(ctx, r), other, st, acc));
        std::swap(acc, other);
    }
    CMCHK(rescale_into(ctx, acc, 2, level, y->dev, st));
    y->level = level - 1, y->ncomp = 2;
    y->scale = x->scale * p->pt_scale / (double)ctx->mod[level];
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
