// Rotary position embedding with the ciphertext extraction fused into it (Sec. 4.2, App. D).
//
// A projection leaves partial sums in every slot that is not an output slot; the element-wise
// layer that follows multiplies by plaintexts that are zero there, so the clean-up costs no level
// of its own.  For q and k that layer is the rotary embedding: with the head-interleaved layout
// slot (e, h, tau) = (e*H + h)*t + tau of Sec. 5.3, the dims 2m and 2m+1 of a head sit H*t slots
// apart, and for token n
//     p0 = cos(theta) on the valid slots,  p1 = sin(theta) on those of even dims,
//     p2 = -sin(theta) on those of odd dims,            theta = n * base^(-2m/E),
//     y  = x p0 + Rot(x p2, +H t) + Rot(x p1, -H t)      (three products, two rotations, one level).
// The appendix prints the single-head case ("rotate by 1" = one block); the signs are read so that
// they fit the left-rotation convention of Sec. 2.1.  The plaintexts are encoded at the scale of
// the prime that the rescale removes, so the ciphertext keeps its scale.
#include <math.h>

#include "kernels.h"

struct cm_rope {
    cm_ctx *ctx = nullptr;
    int S, H, E, t, level, token, tau;
    int step_up, step_dn;      // y = x p0 + Rot(x p2, step_up) + Rot(x p1, step_dn)
    double base;
    u64 *d_pts = nullptr;      // [3][level+1][n], multiplier form
    u64 *d_work = nullptr;     // three ciphertexts
};

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// out_k = a * pt_k for k = 0, 1, 2: the ciphertext is read once
__global__ void k_mul_pt3(u64 *out0, u64 *out1, u64 *out2, const u64 *__restrict__ a, const u64 *__restrict__ pts,
                          const ModC *__restrict__ modc, int limbs, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x, r = blockIdx.y, l = r % limbs;
    const ModC m = modc[l];
    const size_t o = (size_t)r * n + i, po = (size_t)l * n + i, ps = (size_t)limbs * n;
    const u64 v = a[o];
    out0[o] = redc((u128)v * pts[po], m.q, m.qinv);
    out1[o] = redc((u128)v * pts[ps + po], m.q, m.qinv);
    out2[o] = redc((u128)v * pts[2 * ps + po], m.q, m.qinv);
}

extern "C" cm_status cm_rope_create(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t level, int32_t token, int32_t tau,
                                    double base, const int64_t *coeffs, cm_rope **out) {
    if (!ctx || !out || heads < 1 || dim < 2 || token < 0 || !(base > 1.0)) return CM_E_INVAL;
    if (level < 1 || level > ctx->L) return CM_E_LEVEL;
    const int S = ctx->n / 2;
    while (!pow2(heads)) heads++;          // a head count that is not a power of two is padded to the next one
    if (!pow2(dim) || heads * dim > S) return CM_E_LAYOUT;
    const int t = S / (heads * dim);
    if (tau < -1 || tau >= t) return CM_E_LAYOUT;
    cm_rope *r = new (std::nothrow) cm_rope();
    if (!r) return CM_E_NOMEM;
    try {
    r->ctx = ctx, r->S = S, r->H = heads, r->E = dim, r->t = t, r->level = level, r->token = token, r->tau = tau, r->base = base;
    r->step_up = heads * t, r->step_dn = -(heads * t);
    const size_t n = ctx->n, ln = (size_t)(level + 1) * n;
    if (hipMalloc((void **)&r->d_pts, 3 * ln * 8) != hipSuccess || hipMalloc((void **)&r->d_work, 6 * ln * 8) != hipSuccess) {
        cm_rope_destroy(r);
        return CM_E_NOMEM;
    }
    const double scale = (double)ctx->mod[level];
    cm_status s = CM_OK;
    std::vector<double> p[3];
    for (auto &v : p) v.assign(S, 0.0);
    // tau = -1: a group of t tokens, token + r at residue r
    for (int r0 = (tau < 0 ? 0 : tau); r0 < (tau < 0 ? t : tau + 1) && !coeffs; r0++)
        for (int e = 0; e < dim; e++) {
            const double th = (double)(token + (tau < 0 ? r0 : 0)) * pow(base, -2.0 * (double)(e / 2) / (double)dim);
            for (int h = 0; h < heads; h++) {
                const size_t i = ((size_t)e * heads + h) * t + r0;
                p[0][i] = cos(th);
                if (e % 2 == 0) p[1][i] = sin(th);
                else p[2][i] = -sin(th);
            }
        }
    for (int k = 0; k < 3 && s == CM_OK; k++) {
        cm_pt pt;
        pt.dev = r->d_pts + k * ln, pt.mont = 1;
        s = coeffs ? cm_pt_from_coeffs(ctx, coeffs + (size_t)k * n, level, scale, &pt)
                   : cm_encode(ctx, p[k].data(), nullptr, p[k].size(), level, scale, &pt);
    }
    if (s != CM_OK) { cm_rope_destroy(r); return s; }
    *out = r;
    return CM_OK;
    } catch (...) {
        cm_rope_destroy(r);
        return CM_E_NOMEM;
    }
}
// Inner rotation (Sec. 5.4): residue tau of every block of t slots moves to residue (tau + delta) mod t.  The same
// shape as the embedding: p0 = 0, p2 = the residues below t - delta (rotated by -delta), p1 = the others (rotated by
// t - delta); masks encoded at the scale of the prime the rescale removes.
extern "C" cm_status cm_inner_rot_create(cm_ctx *ctx, int32_t t, int32_t delta, int32_t level, const int64_t *coeffs,
                                         cm_rope **out) {
    if (!ctx || !out) return CM_E_INVAL;
    if (level < 1 || level > ctx->L) return CM_E_LEVEL;
    const int S = ctx->n / 2;
    if (!pow2(t) || t < 2 || t > S || delta < 1 || delta >= t) return CM_E_LAYOUT;
    cm_rope *r = new (std::nothrow) cm_rope();
    if (!r) return CM_E_NOMEM;
    try {
    r->ctx = ctx, r->S = S, r->H = 1, r->E = S / t, r->t = t, r->level = level, r->token = 0, r->tau = 0, r->base = 0;
    r->step_up = -delta, r->step_dn = t - delta;
    const size_t n = ctx->n, ln = (size_t)(level + 1) * n;
    if (hipMalloc((void **)&r->d_pts, 3 * ln * 8) != hipSuccess || hipMalloc((void **)&r->d_work, 6 * ln * 8) != hipSuccess) {
        cm_rope_destroy(r);
        return CM_E_NOMEM;
    }
    const double scale = (double)ctx->mod[level];
    std::vector<double> p[3];
    for (auto &v : p) v.assign(S, 0.0);
    for (int i = 0; i < S && !coeffs; i++) p[(i % t) < t - delta ? 2 : 1][i] = 1.0;
    cm_status s = CM_OK;
    for (int k = 0; k < 3 && s == CM_OK; k++) {
        cm_pt pt;
        pt.dev = r->d_pts + k * ln, pt.mont = 1;
        s = coeffs ? cm_pt_from_coeffs(ctx, coeffs + (size_t)k * n, level, scale, &pt)
                   : cm_encode(ctx, p[k].data(), nullptr, p[k].size(), level, scale, &pt);
    }
    if (s != CM_OK) { cm_rope_destroy(r); return s; }
    *out = r;
    return CM_OK;
    } catch (...) {
        cm_rope_destroy(r);
        return CM_E_NOMEM;
    }
}
extern "C" void cm_rope_destroy(cm_rope *r) {
    if (!r) return;
    hipFree(r->d_pts);
    hipFree(r->d_work);
    delete r;
}
extern "C" int32_t cm_rope_steps(const cm_rope *r, int32_t *steps, int32_t cap) {
    if (!r) return 0;
    const int s[2] = {r->step_up, r->step_dn};
    for (int i = 0; i < 2 && i < cap && steps; i++) steps[i] = s[i];
    return 2;
}
extern "C" cm_status cm_rope_apply(cm_ctx *ctx, const cm_evk *evk, const cm_rope *r, const cm_ct *x, cm_ct *y, void *stream) {
    (void)hipGetLastError();          // stale errors of earlier calls are not this call's
    if (!ctx || !evk || !r || r->ctx != ctx || !x || !x->dev || x->ncomp != 2 || !y || !y->dev || y->dev == x->dev ||
        !evk_fits(ctx, evk))
        return CM_E_INVAL;
    if (x->level != r->level) return CM_E_LEVEL;
    CM_TRY
    hipStream_t st = (hipStream_t)stream;
    const int level = r->level, limbs = level + 1;
    const u64 g_up = galois_of_step(ctx, r->step_up), g_dn = galois_of_step(ctx, r->step_dn);
    const u64 *k_up = find_key(evk, g_up), *k_dn = find_key(evk, g_dn);
    if (!k_up || !k_dn) return CM_E_NOKEY;
    const size_t ctw = 2 * (size_t)limbs * ctx->n;
    u64 *a = r->d_work, *b = a + ctw, *c = b + ctw;
    hipLaunchKernelGGL(k_mul_pt3, dim3(ctx->n / 256, 2 * limbs), dim3(256), 0, st, a, c, b, x->dev, r->d_pts, ctx->d_modc, limbs,
                       ctx->n);                                   // a = x p0, c = x p1, b = x p2
    CMCHK(rotate_into(ctx, k_up, b, level, g_up, a, st, a));      // a += Rot(x p2, step_up)
    CMCHK(rotate_into(ctx, k_dn, c, level, g_dn, a, st, a));      // a += Rot(x p1, step_dn)
    CMCHK(rescale_into(ctx, a, 2, level, y->dev, st));
    y->level = level - 1, y->ncomp = 2;
    y->scale = x->scale;                                          // plaintext scale = the prime just removed
    RETURN_LAUNCH_STATUS();
    CM_CATCH
}
