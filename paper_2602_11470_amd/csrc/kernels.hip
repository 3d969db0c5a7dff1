// Element-wise, base-conversion, key-switch and sampling kernels of libcachemir (gfx950).
// Polynomials are [limbs][n] 64-bit words.  "mont" operands are pre-multiplied by 2^64 mod q.
#include "kernels.h"

#define TPB 256
typedef u64 u64x2 __attribute__((ext_vector_type(2)));


// ---- a short list of integers into device memory without a copy or an allocation ---------------
// (the values travel as kernel arguments, so the launch can be captured into a graph)
#define IDX_CHUNK 256
struct IdxChunk { int v[IDX_CHUNK]; };
__global__ void k_set_idx(int *dst, IdxChunk c, int count) {
    const int i = threadIdx.x;
    if (i < count) dst[i] = c.v[i];
}
void launch_set_idx(int *d_dst, const int *h_src, int count, hipStream_t st) {
    for (int base = 0; base < count; base += IDX_CHUNK) {
        IdxChunk c;
        const int m = count - base < IDX_CHUNK ? count - base : IDX_CHUNK;
        for (int i = 0; i < IDX_CHUNK; i++) c.v[i] = i < m ? h_src[base + i] : 0;
        hipLaunchKernelGGL(k_set_idx, dim3(1), dim3(IDX_CHUNK), 0, st, d_dst + base, c, m);
    }
}

// ---- signed integers -> residues -------------------------------------------------------------
__global__ void k_reduce_i64(u64 *out, const long long *coeffs, const int *mod_idx, const ModC *modc, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[mod_idx[l]];
    long long c = coeffs[i];
    u64 a = c < 0 ? (u64)(-(c + 1)) + 1ULL : (u64)c;        // |c| without overflow
    u64 r = redc((u128)to_mont(a, m), m.q, m.qinv);         // |c| mod q
    out[(size_t)l * n + i] = (c < 0 && r) ? m.q - r : r;
}
void launch_reduce_i64(cm_ctx *ctx, u64 *out, const long long *d_coeffs, const int *d_mod_idx, int limbs, hipStream_t st) {
    hipLaunchKernelGGL(k_reduce_i64, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, d_coeffs, d_mod_idx, ctx->d_modc, ctx->n);
}

__global__ void k_to_mont(u64 *data, const int *mod_idx, const ModC *modc, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[mod_idx[l]];
    size_t o = (size_t)l * n + i;
    data[o] = to_mont(data[o], m);
}
void launch_to_mont(cm_ctx *ctx, u64 *data, const int *d_mod_idx, int limbs, hipStream_t st) {
    hipLaunchKernelGGL(k_to_mont, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, data, d_mod_idx, ctx->d_modc, ctx->n);
}
__global__ void k_from_mont(u64 *out, const u64 *in, const int *mod_idx, const ModC *modc, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[mod_idx[l]];
    size_t o = (size_t)l * n + i;
    out[o] = redc((u128)in[o], m.q, m.qinv);
}
void launch_from_mont(cm_ctx *ctx, u64 *out, const u64 *in, const int *d_mod_idx, int limbs, hipStream_t st) {
    hipLaunchKernelGGL(k_from_mont, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, in, d_mod_idx, ctx->d_modc, ctx->n);
}

// ---- ciphertext element-wise ---------------------------------------------------------------------
// rows = ncomp*limbs; row r has modulus index r % limbs
__global__ void k_add(u64 *out, const u64 *a, const u64 *b, const ModC *modc, int limbs, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, r = blockIdx.y;
    u64 q = modc[r % limbs].q;
    size_t o = (size_t)r * n + i;
    out[o] = addmod(a[o], b[o], q);
}
void launch_add(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int ncomp, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, ncomp * limbs, st);
    hipLaunchKernelGGL(k_add, dim3(ctx->n / TPB, ncomp * limbs), dim3(TPB), 0, st, out, a, b, ctx->d_modc, limbs, ctx->n);
}

__global__ void k_mul_pt(u64 *out, const u64 *a, const u64 *pt_mont, const ModC *modc, int limbs, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, r = blockIdx.y;
    const ModC m = modc[r % limbs];
    size_t o = (size_t)r * n + i;
    out[o] = redc((u128)a[o] * pt_mont[(size_t)(r % limbs) * n + i], m.q, m.qinv);
}
void launch_mul_pt(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *pt_mont, int ncomp, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, ncomp * limbs, st);
    hipLaunchKernelGGL(k_mul_pt, dim3(ctx->n / TPB, ncomp * limbs), dim3(TPB), 0, st, out, a, pt_mont, ctx->d_modc, limbs, ctx->n);
}

// out[z][2][limbs][n] = src_z * perm_{g_z}(pt): up to 8 ciphertexts times slot rotations of one
// plaintext (the rotation is the Galois permutation of its evaluation-domain words), one launch
__global__ void k_mul_pt_rot_batch(u64 *__restrict__ out, MulPtBatch b, const u64 *__restrict__ pt_mont,
                                   const ModC *__restrict__ modc, int limbs, int n, int logn) {
    const unsigned i = blockIdx.x * TPB + threadIdx.x;
    const int r = blockIdx.y, z = blockIdx.z, l = r % limbs;
    const ModC m = modc[l];
    const unsigned g = b.g[z];
    const unsigned s = g ? perm_src(i, g, logn) : i;
    out[((size_t)z * 2 * limbs + r) * n + i] = redc((u128)b.src[z][(size_t)r * n + i] * pt_mont[(size_t)l * n + s], m.q, m.qinv);
}
__global__ void k_mul_pt_rot_last(u64 *__restrict__ out, MulPtBatch b, const u64 *__restrict__ pt_mont,
                                  const ModC *__restrict__ modc, int limbs, int n, int logn) {
    const unsigned i = blockIdx.x * TPB + threadIdx.x;
    const int c = blockIdx.y, z = blockIdx.z, l = limbs - 1;
    const ModC m = modc[l];
    const unsigned g = b.g[z];
    const unsigned s = g ? perm_src(i, g, logn) : i;
    out[((size_t)z * 2 + c) * n + i] = redc((u128)b.src[z][((size_t)c * limbs + l) * n + i] * pt_mont[(size_t)l * n + s], m.q, m.qinv);
}
void launch_mul_pt_rot_last(cm_ctx *ctx, u64 *out, const MulPtBatch &b, int cnt, const u64 *pt_mont, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, cnt * 2, st);
    hipLaunchKernelGGL(k_mul_pt_rot_last, dim3(ctx->n / TPB, 2, cnt), dim3(TPB), 0, st, out, b, pt_mont, ctx->d_modc, limbs, ctx->n,
                       ctx->logn);
}
// the same with ONE source for all cnt products: its word is read once and the lane walks over the rotations
__global__ void k_mul_pt_rot_same(u64 *__restrict__ out, MulPtBatch b, int cnt, const u64 *__restrict__ pt_mont,
                                  const ModC *__restrict__ modc, int limbs, int n, int logn) {
    const unsigned i = blockIdx.x * TPB + threadIdx.x;
    const int r = blockIdx.y, l = r % limbs;
    const ModC m = modc[l];
    const u64 v = b.src[0][(size_t)r * n + i];
    for (int z = 0; z < cnt; z++) {
        const unsigned g = b.g[z];
        const unsigned s = g ? perm_src(i, g, logn) : i;
        out[((size_t)z * 2 * limbs + r) * n + i] = redc((u128)v * pt_mont[(size_t)l * n + s], m.q, m.qinv);
    }
}
void launch_mul_pt_rot_batch(cm_ctx *ctx, u64 *out, const MulPtBatch &b, int cnt, const u64 *pt_mont, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, cnt * 2 * limbs, st);
    bool same = cnt > 1;
    for (int z = 1; z < cnt; z++) same = same && b.src[z] == b.src[0];
    if (same) {
        hipLaunchKernelGGL(k_mul_pt_rot_same, dim3(ctx->n / TPB, 2 * limbs), dim3(TPB), 0, st, out, b, cnt, pt_mont, ctx->d_modc,
                           limbs, ctx->n, ctx->logn);
        return;
    }
    hipLaunchKernelGGL(k_mul_pt_rot_batch, dim3(ctx->n / TPB, 2 * limbs, cnt), dim3(TPB), 0, st, out, b, pt_mont, ctx->d_modc,
                       limbs, ctx->n, ctx->logn);
}

// acc (+)= a * pt_mont over ncomp components; accumulate != 0 adds into out
__global__ void k_mac_pt(u64 *out, const u64 *a, const u64 *pt_mont, const ModC *modc, int limbs, int n, int accumulate) {
    int i = blockIdx.x * TPB + threadIdx.x, r = blockIdx.y;
    const ModC m = modc[r % limbs];
    size_t o = (size_t)r * n + i;
    u64 v = redc((u128)a[o] * pt_mont[(size_t)(r % limbs) * n + i], m.q, m.qinv);
    out[o] = accumulate ? addmod(out[o], v, m.q) : v;
}
void launch_mac_pt(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *pt_mont, int ncomp, int limbs, int accumulate, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, ncomp * limbs, st);
    hipLaunchKernelGGL(k_mac_pt, dim3(ctx->n / TPB, ncomp * limbs), dim3(TPB), 0, st, out, a, pt_mont, ctx->d_modc, limbs, ctx->n, accumulate);
}

// Tensor product of two 2-component ciphertexts: (a0 b0, a0 b1 + a1 b0, a1 b1); accumulate adds.
__global__ void k_tensor(u64 *out, const u64 *a, const u64 *b, const ModC *modc, int limbs, int n, int accumulate) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[l];
    size_t o = (size_t)l * n + i, cs = (size_t)limbs * n;
    u64 a0 = to_mont(a[o], m), a1 = to_mont(a[o + cs], m);
    u64 b0 = b[o], b1 = b[o + cs];
    u64 d0 = redc((u128)a0 * b0, m.q, m.qinv);
    u64 d1 = redc((u128)a0 * b1 + (u128)a1 * b0, m.q, m.qinv);     // two products: (T >> 64) < q holds for q < 2^63
    u64 d2 = redc((u128)a1 * b1, m.q, m.qinv);
    if (accumulate) {
        d0 = addmod(d0, out[o], m.q);
        d1 = addmod(d1, out[o + cs], m.q);
        d2 = addmod(d2, out[o + 2 * cs], m.q);
    }
    out[o] = d0;
    out[o + cs] = d1;
    out[o + 2 * cs] = d2;
}
// out[z][3][limbs][n] = a (x) b[z] for cnt ciphertexts b stacked at stride 2*limbs*n: one launch
__global__ void k_tensor_batch(u64 *__restrict__ out, const u64 *__restrict__ a, const u64 *__restrict__ b,
                               const ModC *__restrict__ modc, int limbs, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y, z = blockIdx.z;
    const ModC m = modc[l];
    size_t o = (size_t)l * n + i, cs = (size_t)limbs * n;
    u64 a0 = to_mont(a[o], m), a1 = to_mont(a[o + cs], m);
    const u64 *bz = b + (size_t)z * 2 * cs;
    u64 *oz = out + (size_t)z * 3 * cs;
    u64 b0 = bz[o], b1 = bz[o + cs];
    oz[o] = redc((u128)a0 * b0, m.q, m.qinv);
    oz[o + cs] = redc((u128)a0 * b1 + (u128)a1 * b0, m.q, m.qinv);
    oz[o + 2 * cs] = redc((u128)a1 * b1, m.q, m.qinv);
}
void launch_tensor_batch(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int cnt, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, 3 * limbs * cnt, st);
    hipLaunchKernelGGL(k_tensor_batch, dim3(ctx->n / TPB, limbs, cnt), dim3(TPB), 0, st, out, a, b, ctx->d_modc, limbs, ctx->n);
}
// acc[2][limbs][n] (+)= sum_z src[z] * (pt rotated by g[z]); src stacked at stride 2*limbs*n: one launch, acc written once
__global__ void k_mac_pt_rot_batch(u64 *acc, const u64 *__restrict__ src, MulPtBatch b, int cnt,
                                   const u64 *__restrict__ pt_mont, const ModC *__restrict__ modc, int limbs, int n, int logn,
                                   int accumulate) {
    const unsigned i = blockIdx.x * TPB + threadIdx.x;
    const int r = blockIdx.y, l = r % limbs;
    const ModC m = modc[l];
    const size_t o = (size_t)r * n + i;
    u64 v = accumulate ? acc[o] : 0;
    for (int z = 0; z < cnt; z++) {
        const unsigned g = b.g[z];
        const unsigned s = g ? perm_src(i, g, logn) : i;
        v = addmod(v, redc((u128)src[(size_t)z * 2 * limbs * n + o] * pt_mont[(size_t)l * n + s], m.q, m.qinv), m.q);
    }
    acc[o] = v;
}
void launch_mac_pt_rot_batch(cm_ctx *ctx, u64 *acc, const u64 *src, const MulPtBatch &b, int cnt, const u64 *pt_mont,
                             int limbs, int accumulate, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, cnt * 2 * limbs, st);
    hipLaunchKernelGGL(k_mac_pt_rot_batch, dim3(ctx->n / TPB, 2 * limbs), dim3(TPB), 0, st, acc, src, b, cnt, pt_mont,
                       ctx->d_modc, limbs, ctx->n, ctx->logn, accumulate);
}
// FP64 modular products for limbs whose modulus is below 2^50 (the arithmetic is explained at k_vmm_mac_lds)
struct MacFp {
    double q, qinv;
    __device__ __forceinline__ double mulmod(double y, double a, double aq) const {
        double h = y * a;
        double l = __builtin_fma(y, a, -h);
        double c = __builtin_rint(y * aq);
        return __builtin_fma(-c, q, h) + l;
    }
    __device__ __forceinline__ double norm(double x) const { return __builtin_fma(-__builtin_rint(x * qinv), q, x); }
    __device__ __forceinline__ static double from_u64(u64 raw) {                 // raw < 2^52
        return __longlong_as_double((long long)(raw | 0x4330000000000000ULL)) - 4503599627370496.0;
    }
    __device__ __forceinline__ u64 canon(double v) const {                       // |v| < 2^52 -> [0, q)
        double r = __builtin_fma(-__builtin_floor(v * qinv), q, v);
        r = r < 0.0 ? r + q : r;
        r = r >= q ? r - q : r;
        return (u64)__double_as_longlong(r + 4503599627370496.0) & 0x000FFFFFFFFFFFFFULL;
    }
};
// out[z][3][limbs][n] = sum_{j < cnt} a[j] (x) b[z*gs + j*ts]: a and b stacked at stride 2*limbs*n (gs, ts = the distance of
// groups and of the terms of a group in b, in ciphertexts); every output written once.
// On limbs below 2^50 the four products per term run in FP64 (no multiplier form needed), sums renormalised every two terms.
__global__ void k_tensor_sum(u64 *__restrict__ out, const u64 *__restrict__ a, const u64 *__restrict__ b,
                             const ModC *__restrict__ modc, const FpQ *__restrict__ fpq, int limbs, int n, int cnt, int gs,
                             int ts) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y, z = blockIdx.z;
    const ModC m = modc[l];
    const size_t o = (size_t)l * n + i, cs = (size_t)limbs * n;
    const FpQ fq = fpq[l];
    if (fq.q != 0.0) {
        const MacFp F{fq.q, fq.qinv};
        double d0 = 0.0, d1 = 0.0, d2 = 0.0;
        for (int j = 0; j < cnt; j++) {
            const u64 *aj = a + (size_t)j * 2 * cs, *bj = b + ((size_t)z * gs + (size_t)j * ts) * 2 * cs;
            const double a0 = MacFp::from_u64(aj[o]), a1 = MacFp::from_u64(aj[o + cs]);
            const double b0 = MacFp::from_u64(__builtin_nontemporal_load(bj + o));
            const double b1 = MacFp::from_u64(__builtin_nontemporal_load(bj + o + cs));
            const double b0q = b0 * F.qinv, b1q = b1 * F.qinv;
            d0 += F.mulmod(a0, b0, b0q);
            d1 += F.mulmod(a0, b1, b1q) + F.mulmod(a1, b0, b0q);
            d2 += F.mulmod(a1, b1, b1q);
            if (j & 1) d0 = F.norm(d0), d1 = F.norm(d1), d2 = F.norm(d2);
        }
        u64 *oz = out + (size_t)z * 3 * cs;
        oz[o] = F.canon(d0);
        oz[o + cs] = F.canon(d1);
        oz[o + 2 * cs] = F.canon(d2);
        return;
    }
    u64 d0 = 0, d1 = 0, d2 = 0;
    for (int j = 0; j < cnt; j++) {
        const u64 *aj = a + (size_t)j * 2 * cs, *bj = b + ((size_t)z * gs + (size_t)j * ts) * 2 * cs;
        const u64 a0 = to_mont(aj[o], m), a1 = to_mont(aj[o + cs], m);
        const u64 b0 = __builtin_nontemporal_load(bj + o), b1 = __builtin_nontemporal_load(bj + o + cs);
        d0 = addmod(d0, redc((u128)a0 * b0, m.q, m.qinv), m.q);
        d1 = addmod(d1, redc((u128)a0 * b1 + (u128)a1 * b0, m.q, m.qinv), m.q);
        d2 = addmod(d2, redc((u128)a1 * b1, m.q, m.qinv), m.q);
    }
    u64 *oz = out + (size_t)z * 3 * cs;
    oz[o] = d0;
    oz[o + cs] = d1;
    oz[o + 2 * cs] = d2;
}
// The same sums with the cnt <= TS_MAX_CNT ciphertexts a[j] held in registers (FP64 limbs only) while the lane runs over
// all groups: a is read once instead of once per group, which is half of the traffic when a does not fit the caches.
#define TS_MAX_CNT 16
__global__ __launch_bounds__(TPB) void k_tensor_sum_stationary(u64 *__restrict__ out, const u64 *__restrict__ a,
                                                               const u64 *__restrict__ b, const FpQ *__restrict__ fpq,
                                                               int limbs, int n, int cnt, int groups, int gs, int ts) {
    const int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const FpQ fq = fpq[l];
    const MacFp F{fq.q, fq.qinv};
    const size_t o = (size_t)l * n + i, cs = (size_t)limbs * n;
    double a0[TS_MAX_CNT], a1[TS_MAX_CNT];
#pragma unroll
    for (int j = 0; j < TS_MAX_CNT; j++) {
        a0[j] = j < cnt ? MacFp::from_u64(a[(size_t)j * 2 * cs + o]) : 0.0;
        a1[j] = j < cnt ? MacFp::from_u64(a[(size_t)j * 2 * cs + cs + o]) : 0.0;
    }
    for (int z = 0; z < groups; z++) {
        double d0 = 0.0, d1 = 0.0, d2 = 0.0;
        // Eight terms at a time: their sixteen words are requested before the first is used.  Terms at or past cnt read
        // term 0's words again (a valid address) and multiply them by a zero, so no load sits behind a branch.
#pragma unroll
        for (int jc = 0; jc < TS_MAX_CNT; jc += 8) {
            if (jc < cnt) {
                u64 r0[8], r1[8];
#pragma unroll
                for (int jj = 0; jj < 8; jj++) {
                    const int j = jc + jj < cnt ? jc + jj : 0;
                    const u64 *bj = b + ((size_t)z * gs + (size_t)j * ts) * 2 * cs;
                    r0[jj] = __builtin_nontemporal_load(bj + o), r1[jj] = __builtin_nontemporal_load(bj + o + cs);
                }
#pragma unroll
                for (int jj = 0; jj < 8; jj++) {
                    const int j = jc + jj;
                    const double b0 = MacFp::from_u64(r0[jj]), b1 = MacFp::from_u64(r1[jj]);
                    const double b0q = b0 * F.qinv, b1q = b1 * F.qinv;
                    d0 += F.mulmod(a0[j], b0, b0q);
                    d1 += F.mulmod(a0[j], b1, b1q) + F.mulmod(a1[j], b0, b0q);
                    d2 += F.mulmod(a1[j], b1, b1q);
                    if (jj & 1) d0 = F.norm(d0), d1 = F.norm(d1), d2 = F.norm(d2);
                }
            }
        }
        u64 *oz = out + (size_t)z * 3 * cs;
        oz[o] = F.canon(d0);
        oz[o + cs] = F.canon(d1);
        oz[o + 2 * cs] = F.canon(d2);
    }
}
void launch_tensor_sum(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int cnt, int groups, int limbs, hipStream_t st,
                       int group_stride, int term_stride) {
    const int gs = group_stride ? group_stride : cnt, ts = term_stride ? term_stride : 1;
    Prof prof_(ctx, CM_K_ELEMENTWISE, 3 * limbs * groups, st);
    bool all_fp = true;
    for (int l = 0; l < limbs; l++) all_fp = all_fp && ctx->mod[l] < (1ULL << 50);
    if (all_fp && cnt <= TS_MAX_CNT && groups > 1) {
        hipLaunchKernelGGL(k_tensor_sum_stationary, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, a, b, ctx->d_fpq, limbs, ctx->n,
                           cnt, groups, gs, ts);
        return;
    }
    hipLaunchKernelGGL(k_tensor_sum, dim3(ctx->n / TPB, limbs, groups), dim3(TPB), 0, st, out, a, b, ctx->d_modc, ctx->d_fpq, limbs, ctx->n,
                       cnt, gs, ts);
}
void launch_tensor(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int limbs, int accumulate, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, 3 * limbs, st);
    hipLaunchKernelGGL(k_tensor, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, a, b, ctx->d_modc, limbs, ctx->n, accumulate);
}

// Galois map on evaluation-domain rows (a pure permutation); rows = ncomp*limbs
__global__ void k_automorphism(u64 *out, const u64 *in, int n, int logn, unsigned g) {
    unsigned i = blockIdx.x * TPB + threadIdx.x;
    size_t r = blockIdx.y;
    out[r * n + i] = in[r * n + perm_src(i, g, logn)];
}
void launch_automorphism(cm_ctx *ctx, u64 *out, const u64 *in, int rows, u64 g, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, rows, st);
    hipLaunchKernelGGL(k_automorphism, dim3(ctx->n / TPB, rows), dim3(TPB), 0, st, out, in, ctx->n, ctx->logn, (unsigned)g);
}

// Sum of products d * w with d below 2^50 held as two 25-bit halves (d = d0 + 2^25 d1) and w any 64-bit word: four
// 32 x 32 -> 64-bit multiply-adds into four accumulators that cannot overflow for up to 16 terms (each term is below
// 2^57), so a product costs four instructions and no carry chain; the accumulators are combined once per sum.  The
// generic form (64 x 64 -> 128 with carries, about ten instructions) stays for the 60-bit moduli.
struct Acc50 {
    u64 t00 = 0, t01 = 0, t10 = 0, t11 = 0;
    __device__ __forceinline__ void mac(unsigned d0, unsigned d1, u64 w) {
        const unsigned w0 = (unsigned)w, w1 = (unsigned)(w >> 32);
        t00 += (u64)d0 * w0, t01 += (u64)d0 * w1, t10 += (u64)d1 * w0, t11 += (u64)d1 * w1;
    }
    __device__ __forceinline__ u128 total() const {
        return (u128)t00 + ((u128)t01 << 32) + ((u128)t10 << 25) + ((u128)t11 << 57);
    }
};
#define LOW25 0x1FFFFFFu
// converted limbs are written with non-temporal stores (next read by the transform kernel, after the whole launch)
#define CONV_ST(ptr, val) __builtin_nontemporal_store((u64)(val), (ptr))
// ---- fast base conversion ----------------------------------------------------------------------
// in rows in_rows[m] (coefficient domain, residues under src moduli) -> out rows out_rows[r]:
//   y_m = a_m * inv_hat_m mod q_m;  out_r = sum_m y_m * hat_{m,r} mod q_r   (no correction term)
// blockIdx.z = batch item: table (z % tab_period)*tab_step, input at (z / in_group)*in_stride,
// output at z*out_stride (the digits of a raise use one table each and share the input; the two
// components of a ModDown share the table; a raise of several polynomials runs its digits over
// z % beta and its polynomials over z / beta).  blockIdx.y = group of CONV_TG targets; the cheap y_m are recomputed per group so
// that a conversion fills the machine.  If own_src is given, group 0 also copies the source rows
// of own_src (the evaluation-domain input) to the same rows of the output.
// NS = compile-time bound on the source count: the table rows past ns are all zero (a zero inverse, a zero modulus, zero
// weights, input row 0), so the arithmetic runs unconditionally over NS rows and every load of a lane is in flight at once
// instead of one load-wait-use chain per source.
template <int CONV_TG, int NS>
__global__ __launch_bounds__(TPB) void k_base_conv(u64 *__restrict__ out, const u64 *__restrict__ in,
                                                   const ConvDev *__restrict__ tabs, int tab_step, int tab_period,
                                                   int in_group, int n, size_t in_stride, size_t out_stride,
                                                   const u64 *__restrict__ own_src, size_t own_stride, unsigned own_g,
                                                   int logn) {
    const int i = blockIdx.x * TPB + threadIdx.x;
    const ConvDev &t = tabs[(blockIdx.z % tab_period) * tab_step];
    const int ns = t.ns, nt = t.nt;
    const int r0 = blockIdx.y * CONV_TG;
    if (r0 >= nt) return;
    in += (blockIdx.z / in_group) * in_stride;
    out += blockIdx.z * out_stride;
    u64 x[NS], y[NS];
#pragma unroll
    for (int m = 0; m < NS; m++) x[m] = in[(size_t)t.in_rows[m] * n + i];
    if (own_src && r0 == 0) {
        own_src += (blockIdx.z / in_group) * own_stride;
        const unsigned s = own_g ? perm_src((unsigned)i, own_g, logn) : (unsigned)i;
        u64 o[NS];
#pragma unroll
        for (int m = 0; m < NS; m++) o[m] = own_src[(size_t)t.in_rows[m] * n + s];
#pragma unroll
        for (int m = 0; m < NS; m++)
            if (m < ns) out[(size_t)t.in_rows[m] * n + i] = o[m];
    }
#pragma unroll
    for (int m = 0; m < NS; m++) y[m] = mul_shoup(x[m], t.inv_hat[m], t.inv_hat_sh[m], t.src_q[m]);
    // source moduli below 2^50 (the digits of a ModUp): carry-free split products, four multiply-adds per term
    u64 qmax = 0;
#pragma unroll
    for (int m = 0; m < NS; m++) qmax = t.src_q[m] > qmax ? t.src_q[m] : qmax;
    if (qmax < (1ULL << 50)) {
        unsigned y0[NS], y1[NS];
#pragma unroll
        for (int m = 0; m < NS; m++) y0[m] = (unsigned)y[m] & LOW25, y1[m] = (unsigned)(y[m] >> 25);
#pragma unroll
        for (int rr = 0; rr < CONV_TG; rr++) {
            const int r = r0 + rr;
            if (r < nt) {
                Acc50 acc;
#pragma unroll
                for (int m = 0; m < NS; m++) acc.mac(y0[m], y1[m], t.hat_mont[m * nt + r]);
                CONV_ST(out + (size_t)t.out_rows[r] * n + i, redc(acc.total(), t.dst_q[r], t.dst_qinv[r]));
            }
        }
        return;
    }
#pragma unroll
    for (int rr = 0; rr < CONV_TG; rr++) {
        const int r = r0 + rr;
        if (r < nt) {
            u128 acc = 0;
#pragma unroll
            for (int m = 0; m < NS; m++) acc += (u128)y[m] * t.hat_mont[m * nt + r];
            CONV_ST(out + (size_t)t.out_rows[r] * n + i, redc(acc, t.dst_q[r], t.dst_qinv[r]));
        }
    }
}
void launch_base_conv(cm_ctx *ctx, const ConvDev *d_tabs, int batch, int tab_step, int max_nt, u64 *out, const u64 *in,
                      size_t in_stride, size_t out_stride, const u64 *own_src, u64 own_g, hipStream_t st, int tab_period,
                      int in_group, size_t own_stride) {
    if (tab_period <= 0) tab_period = batch;
    Prof prof_(ctx, CM_K_BASE_CONV, batch * max_nt, st);
    // 8 targets per lane (measured best of 2 / 4 / 8 / 12 / 24 at the benchmark's shapes); the source bound is the larger
    // of the digit size and the special prime count, rounded up to an instantiated one
    const int TG = 8, ns = ctx->alpha > ctx->K ? ctx->alpha : ctx->K;
    const dim3 grid(ctx->n / TPB, (max_nt + TG - 1) / TG, batch);
#define CONV_LAUNCH(NS_)                                                                                                 \
    hipLaunchKernelGGL((k_base_conv<8, NS_>), grid, dim3(TPB), 0, st, out, in, d_tabs, tab_step, tab_period, in_group, ctx->n, \
                       in_stride, out_stride, own_src, own_stride, (unsigned)own_g, ctx->logn)
    if (ns <= 1) CONV_LAUNCH(1);
    else if (ns <= 2) CONV_LAUNCH(2);
    else if (ns <= 4) CONV_LAUNCH(4);
    else if (ns <= 6) CONV_LAUNCH(6);
    else CONV_LAUNCH(8);
#undef CONV_LAUNCH
}

// ---- evaluation-key inner product ------------------------------------------------------------------
// u0[r] = sum_j dig[j][r] * evk[j][0][mod(r)],  u1 likewise with evk[j][1]; r over the level's
// extended basis.  With g != 0 the digits are read through the Galois permutation (hoisted
// rotations).  Two adjacent coefficients per lane (16-byte accesses); the permutation keeps
// aligned pairs together (it maps i^1 to src^1).
// `extra` may be the output itself (a running sum): every lane reads its own words before it writes them.
// The counter-based generator (its finaliser; the streams are defined with the samplers below).
#define GOLD 0x9E3779B97F4A7C15ULL
__host__ __device__ __forceinline__ u64 mix64(u64 z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
// An evaluation key in HBM is its b half only: b_j in multiplier form, [digit][nmod][n], followed by the [digit][nmod]
// keys of the generator streams of a_j.  The uniform half is drawn directly in the evaluation domain, so word i of
// limb mi of a_j is draw i of that stream (rejected at or above bound = q floor(2^64/q), then taken mod q): the inner
// products regenerate it instead of reading it, which takes a third off their traffic.  The draw enters the sums as
// the raw 64-bit word v (v = a mod q): sum_j d_j v_j < beta q 2^64 fits 128 bits, REDC gives (sum 2^-64) mod q below
// (beta + 1) q, and a second REDC against 2^128 mod q gives sum mod q in [0, q) -- two reductions per output instead of
// one per key word.  ctr_gold = (i + 1) GOLD is the counter term of attempt 0, shared by all digits of a lane.
__device__ __forceinline__ u64 evk_a_draw(u64 stream_key, u64 ctr_gold, unsigned i, u64 bound) {
    u64 v = mix64(stream_key + ctr_gold);
    for (u64 att = 1; v >= bound; att++) v = mix64(stream_key + (((att << 32) | (u64)i) + 1) * GOLD);
    return v;
}
__device__ __forceinline__ u64 redc_raw(u128 T, const ModC &m) {
    return redc((u128)redc(T, m.q, m.qinv) * m.r2, m.q, m.qinv);
}
// Where the two words of a_j for positions (i, i + 1) of limb mi come from.  Keys generated with both halves stored
// carry a_j in multiplier form like b_j (word offset a_off inside the key): the kernels read it, one REDC per sum.
// Otherwise it is regenerated from its stream (raw draws, two REDCs per sum).  Both give the same residues.
struct EvkA {
    size_t a_off;     // 0: regenerate
    int kdig;         // digits of a full key: the stream keys start at kdig * nmod * n
};
template <bool SA>
__device__ __forceinline__ ulonglong2 evk_a_words(const u64 *__restrict__ key, const EvkA ea, int nmod, int n, int j, int mi,
                                                  unsigned i, u64 cg0, u64 cg1, u64 bound) {
    ulonglong2 r;
    if (SA) {
        const u64 *ka = key + ea.a_off + ((size_t)j * nmod + mi) * n + i;
        r.x = __builtin_nontemporal_load(ka), r.y = __builtin_nontemporal_load(ka + 1);
    } else {
        const u64 sk_ = key[(size_t)ea.kdig * nmod * n + (size_t)j * nmod + mi];
        r.x = evk_a_draw(sk_, cg0, i, bound), r.y = evk_a_draw(sk_, cg1, i + 1, bound);
    }
    return r;
}
template <bool SA>
__device__ __forceinline__ u64 evk_a_reduce(u128 T, const ModC &m) {
    return SA ? redc(T, m.q, m.qinv) : redc_raw(T, m);
}
static EvkA evk_a_of(const cm_ctx *ctx) {
    return EvkA{ctx->evk_stored_a ? evk_a_offset(ctx) : 0, (ctx->L + ctx->alpha) / ctx->alpha};
}
template <bool SA>
__global__ __launch_bounds__(TPB) void k_inner_product(u64 *u0, u64 *u1,
                                                       const u64 *__restrict__ dig, const u64 *__restrict__ evk,
                                                       const ModC *__restrict__ modc,
                                int beta, int ext, int level, int L, int nmod, int n, int logn, unsigned g,
                                const u64 *__restrict__ c0, const u64 *__restrict__ pmont, const u64 *extra, EvkA eva,
                                const u64 *__restrict__ ubound) {
    unsigned i2 = (blockIdx.x * TPB + threadIdx.x) * 2;
    int r = blockIdx.y;
    int mi = r <= level ? r : L + 1 + (r - level - 1);
    const ModC m = modc[mi];
    unsigned src = g ? perm_src(i2, g, logn) : i2;
    unsigned base = src & ~1u;
    bool swap = src & 1u;
    const u64 bound = ubound[mi], cg0 = ((u64)i2 + 1) * GOLD, cg1 = cg0 + GOLD;
    u128 a0 = 0, a1 = 0, b0 = 0, b1 = 0;
    for (int j = 0; j < beta; j++) {
        ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(dig + ((size_t)j * ext + r) * n + base);
        u64 dx = swap ? d.y : d.x, dy = swap ? d.x : d.y;
        const u64 *kb = evk + ((size_t)j * nmod + mi) * n + i2;
        // the key is streamed once: non-temporal, so that the raised digits (re-read by every
        // hoisted rotation) are the lines that stay in the last-level cache
        ulonglong2 eb;
        eb.x = __builtin_nontemporal_load(kb), eb.y = __builtin_nontemporal_load(kb + 1);
        const ulonglong2 ea = evk_a_words<SA>(evk, eva, nmod, n, j, mi, i2, cg0, cg1, bound);
        b0 += (u128)dx * eb.x;
        b1 += (u128)dy * eb.y;
        a0 += (u128)dx * ea.x;
        a1 += (u128)dy * ea.y;
    }
    if (c0 && r <= level) {           // + P * sigma_g(c0): the rotation stays in the extended basis
        ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(c0 + (size_t)r * n + base);
        const u64 pm = pmont[r];
        b0 += (u128)(swap ? d.y : d.x) * pm;
        b1 += (u128)(swap ? d.x : d.y) * pm;
    }
    size_t o = (size_t)r * n + i2;
    ulonglong2 r0 = make_ulonglong2(redc(b0, m.q, m.qinv), redc(b1, m.q, m.qinv));
    ulonglong2 r1 = make_ulonglong2(evk_a_reduce<SA>(a0, m), evk_a_reduce<SA>(a1, m));
    if (extra) {                      // + a sum already in the extended basis, [2][ext][n]
        ulonglong2 e0 = *reinterpret_cast<const ulonglong2 *>(extra + o);
        ulonglong2 e1 = *reinterpret_cast<const ulonglong2 *>(extra + (size_t)ext * n + o);
        r0.x = addmod(r0.x, e0.x, m.q), r0.y = addmod(r0.y, e0.y, m.q);
        r1.x = addmod(r1.x, e1.x, m.q), r1.y = addmod(r1.y, e1.y, m.q);
    }
    *reinterpret_cast<ulonglong2 *>(u0 + o) = r0;
    *reinterpret_cast<ulonglong2 *>(u1 + o) = r1;
}
// Several inner products in one launch: blockIdx.z = output; output z sums nsum consecutive items
// (each with its own digits, key, Galois element and optional c0) and an optional addend.
template <bool SA>
__global__ __launch_bounds__(TPB) void k_inner_product_batch(IpBatch b, const ModC *__restrict__ modc, int beta, int ext,
                                                             int level, int L, int nmod, int n, int logn,
                                                             const u64 *__restrict__ pmont, EvkA eva,
                                                             const u64 *__restrict__ ubound) {
    // Workgroups go to the eight XCDs round-robin by their linear index.  The rotated reads of the digits gather over
    // a whole limb, and every key of a sum gathers over the same limb again: with a limb's workgroups on ONE XCD (each
    // XCD takes a contiguous eighth of the (limb, block) sequence) those re-reads can hit that XCD's L2.
    unsigned bx = blockIdx.x;
    int r = blockIdx.y;
    if (gridDim.x % 8 == 0) {
        const unsigned lin = blockIdx.x + gridDim.x * blockIdx.y, per = gridDim.x * gridDim.y / 8;
        const unsigned v = (lin & 7u) * per + (lin >> 3);
        bx = v % gridDim.x, r = v / gridDim.x;
    }
    const unsigned i2 = (bx * TPB + threadIdx.x) * 2;
    const int z = blockIdx.z;
    const int mi = r <= level ? r : L + 1 + (r - level - 1);
    const ModC m = modc[mi];
    const size_t o = (size_t)r * n + i2;
    const u64 bound = ubound[mi], cg0 = ((u64)i2 + 1) * GOLD, cg1 = cg0 + GOLD;
    ulonglong2 r0 = make_ulonglong2(0, 0), r1 = make_ulonglong2(0, 0);
    if (b.extra[z]) {
        r0 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + o);
        r1 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + (size_t)ext * n + o);
    }
    for (int s = 0; s < b.nsum; s++) {
        const IpItem it = b.it[z * b.nsum + s];
        const unsigned src = it.g ? perm_src(i2, it.g, logn) : i2;
        const unsigned base = src & ~1u;
        const bool swap = src & 1u;
        u128 a0 = 0, a1 = 0, b0 = 0, b1 = 0;
        for (int j = 0; j < beta; j++) {
            ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(it.dig + ((size_t)j * ext + r) * n + base);
            u64 dx = swap ? d.y : d.x, dy = swap ? d.x : d.y;
            const u64 *kb = it.key + ((size_t)j * nmod + mi) * n + i2;
            ulonglong2 eb;
            eb.x = __builtin_nontemporal_load(kb), eb.y = __builtin_nontemporal_load(kb + 1);
            const ulonglong2 ea = evk_a_words<SA>(it.key, eva, nmod, n, j, mi, i2, cg0, cg1, bound);
            b0 += (u128)dx * eb.x;
            b1 += (u128)dy * eb.y;
            a0 += (u128)dx * ea.x;
            a1 += (u128)dy * ea.y;
        }
        if (it.c0 && it.c0_ext) {            // a first component that never left the extended basis
            ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(it.c0 + (size_t)r * n + base);
            r0.x = addmod(r0.x, swap ? d.y : d.x, m.q), r0.y = addmod(r0.y, swap ? d.x : d.y, m.q);
        } else if (it.c0 && r <= level) {
            ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(it.c0 + (size_t)r * n + base);
            const u64 pm = pmont[r];
            b0 += (u128)(swap ? d.y : d.x) * pm;
            b1 += (u128)(swap ? d.x : d.y) * pm;
        }
        r0.x = addmod(r0.x, redc(b0, m.q, m.qinv), m.q), r0.y = addmod(r0.y, redc(b1, m.q, m.qinv), m.q);
        r1.x = addmod(r1.x, evk_a_reduce<SA>(a0, m), m.q), r1.y = addmod(r1.y, evk_a_reduce<SA>(a1, m), m.q);
    }
    *reinterpret_cast<ulonglong2 *>(b.out[z] + o) = r0;
    *reinterpret_cast<ulonglong2 *>(b.out[z] + (size_t)ext * n + o) = r1;
}
// The same key applied to nz digit arrays: a lane keeps its key words in registers and runs over the
// arrays, so the key is read from HBM once per launch.  With g != 0 the digits (and the optional
// it[z].c0, a first component already in the extended basis, added as it is) are read through the
// Galois map; extra[z] ([2][ext][n], may be out[z] itself) is added, which lets several launches with
// different keys accumulate into one output.
#define IP_SHARED_MAX_BETA 8
template <bool SA>
__global__ __launch_bounds__(TPB) void k_inner_product_shared_key(IpBatch b, const ModC *__restrict__ modc, int beta,
                                                                  int ext, int level, int L, int nmod, int n, int logn,
                                                                  unsigned g, EvkA eva, const u64 *__restrict__ ubound) {
    const unsigned i2 = (blockIdx.x * TPB + threadIdx.x) * 2;
    const int r = blockIdx.y;
    const int mi = r <= level ? r : L + 1 + (r - level - 1);
    const ModC m = modc[mi];
    const size_t o = (size_t)r * n + i2;
    const unsigned src = g ? perm_src(i2, g, logn) : i2;
    const unsigned base = src & ~1u;
    const bool swap = src & 1u;
    ulonglong2 eb[IP_SHARED_MAX_BETA], ea[IP_SHARED_MAX_BETA];
    const u64 *key = b.it[0].key;
    const u64 bound = ubound[mi], cg0 = ((u64)i2 + 1) * GOLD, cg1 = cg0 + GOLD;
#pragma unroll
    for (int j = 0; j < IP_SHARED_MAX_BETA; j++) {
        if (j < beta) {
            const u64 *kb = key + ((size_t)j * nmod + mi) * n + i2;
            eb[j].x = __builtin_nontemporal_load(kb), eb[j].y = __builtin_nontemporal_load(kb + 1);
            ea[j] = evk_a_words<SA>(key, eva, nmod, n, j, mi, i2, cg0, cg1, bound);
        }
    }
    for (int z = 0; z < b.nz; z++) {
        const u64 *dig = b.it[z].dig;
        u128 a0 = 0, a1 = 0, b0 = 0, b1 = 0;
#pragma unroll
        for (int j = 0; j < IP_SHARED_MAX_BETA; j++) {
            if (j < beta) {
                ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(dig + ((size_t)j * ext + r) * n + base);
                const u64 dx = swap ? d.y : d.x, dy = swap ? d.x : d.y;
                b0 += (u128)dx * eb[j].x;
                b1 += (u128)dy * eb[j].y;
                a0 += (u128)dx * ea[j].x;
                a1 += (u128)dy * ea[j].y;
            }
        }
        ulonglong2 r0 = make_ulonglong2(redc(b0, m.q, m.qinv), redc(b1, m.q, m.qinv));
        ulonglong2 r1 = make_ulonglong2(evk_a_reduce<SA>(a0, m), evk_a_reduce<SA>(a1, m));
        if (b.it[z].c0) {
            ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(b.it[z].c0 + (size_t)r * n + base);
            r0.x = addmod(r0.x, swap ? d.y : d.x, m.q), r0.y = addmod(r0.y, swap ? d.x : d.y, m.q);
        }
        if (b.extra[z]) {
            ulonglong2 e0 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + o);
            ulonglong2 e1 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + (size_t)ext * n + o);
            r0.x = addmod(r0.x, e0.x, m.q), r0.y = addmod(r0.y, e0.y, m.q);
            r1.x = addmod(r1.x, e1.x, m.q), r1.y = addmod(r1.y, e1.y, m.q);
        }
        *reinterpret_cast<ulonglong2 *>(b.out[z] + o) = r0;
        *reinterpret_cast<ulonglong2 *>(b.out[z] + (size_t)ext * n + o) = r1;
    }
}
void launch_inner_product_shared_key(cm_ctx *ctx, const IpBatch &b, int beta, int level, hipStream_t st, u64 g) {
    int ext = level + 1 + ctx->K;
    if (beta > IP_SHARED_MAX_BETA) {          // more digits than a lane keeps: the general batch kernel, one output per array
        IpBatch c = b;
        c.nsum = 1;
        for (int z = 0; z < b.nz; z++) c.it[z].key = b.it[0].key, c.it[z].g = (unsigned)g, c.it[z].c0_ext = c.it[z].c0 ? 1 : 0;
        launch_inner_product_batch(ctx, c, beta, level, st);
        return;
    }
    Prof prof_(ctx, CM_K_INNER_PRODUCT, b.nz, st);
    if (ctx->evk_stored_a)
        hipLaunchKernelGGL(k_inner_product_shared_key<true>, dim3(ctx->n / (2 * TPB), ext), dim3(TPB), 0, st, b, ctx->d_modc, beta,
                           ext, level, ctx->L, ctx->nmod, ctx->n, ctx->logn, (unsigned)g, evk_a_of(ctx), ctx->d_ubound);
    else
        hipLaunchKernelGGL(k_inner_product_shared_key<false>, dim3(ctx->n / (2 * TPB), ext), dim3(TPB), 0, st, b, ctx->d_modc, beta,
                           ext, level, ctx->L, ctx->nmod, ctx->n, ctx->logn, (unsigned)g, evk_a_of(ctx), ctx->d_ubound);
}
// One digit array, many keys, one output per key (the hoisted rotations of ONE ciphertext, each kept on its own): a lane
// keeps the digit words of two SOURCE positions (and the first component's) in registers and walks over the keys; for
// key a it writes its result at the position the Galois map sends its source to (the inverse map; pairs go to pairs,
// aligned runs of 64 to aligned runs of 64, so key reads and result writes stay coalesced).  Same sums as
// k_inner_product_batch, but the digits are read once per IP_FAN_CHUNK keys instead of once per key.
#define IP_FAN_CHUNK 8
template <bool SA>
__global__ __launch_bounds__(TPB) void k_inner_product_fanout(IpFan f, const u64 *__restrict__ dig, const u64 *__restrict__ c0,
                                                              int c0_ext, const ModC *__restrict__ modc, int beta, int ext,
                                                              int level, int L, int nmod, int n, int logn,
                                                              const u64 *__restrict__ pmont, EvkA eva,
                                                              const u64 *__restrict__ ubound) {
    // The key chunks of one (limb, block) read the same digits: they are given consecutive places in the sequence of
    // ONE XCD (workgroups go to the XCDs round-robin by linear index), so that the digits come from HBM once and from
    // that XCD's L2 for the other chunks.
    unsigned bx = blockIdx.x, bz = blockIdx.z;
    int r = blockIdx.y;
    if (gridDim.x % 8 == 0) {
        const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), s = lin >> 3, xs = gridDim.x / 8;
        bz = s % gridDim.z;
        const unsigned rest = s / gridDim.z;
        bx = (lin & 7u) + 8u * (rest % xs), r = rest / xs;
    }
    const unsigned s2 = (bx * TPB + threadIdx.x) * 2;
    const int mi = r <= level ? r : L + 1 + (r - level - 1);
    const ModC m = modc[mi];
    const u64 bound = ubound[mi];
    const bool small = m.q < (1ULL << 50);
    ulonglong2 d[IP_SHARED_MAX_BETA];
#pragma unroll
    for (int j = 0; j < IP_SHARED_MAX_BETA; j++)
        if (j < beta) d[j] = *reinterpret_cast<const ulonglong2 *>(dig + ((size_t)j * ext + r) * n + s2);
    // the first component's contribution to the first output component: sigma(c0) as it is (extended basis) or
    // P sigma(c0) on the ciphertext limbs
    ulonglong2 cv = make_ulonglong2(0, 0);
    const bool have_c0 = c0 && (c0_ext || r <= level);
    if (have_c0) {
        cv = *reinterpret_cast<const ulonglong2 *>(c0 + (size_t)r * n + s2);
        if (!c0_ext) {
            const u64 pm = pmont[r];
            cv.x = redc((u128)cv.x * pm, m.q, m.qinv), cv.y = redc((u128)cv.y * pm, m.q, m.qinv);
        }
    }
    const int a_end = min(f.n, (int)(bz + 1) * IP_FAN_CHUNK);
    // The generator stream keys of this chunk's (key, digit) pairs: lane 8 a' + j of every wave fetches one, and the loop
    // below broadcasts it with a lane read, so that no draw waits for a load of its own.
    u64 my_sk = 0;
    if (!SA) {
        const int la = (threadIdx.x & 63) >> 3, lj = threadIdx.x & 7;
        static_assert(IP_FAN_CHUNK * IP_SHARED_MAX_BETA == 64, "one lane per (key, digit) of a chunk");
        if ((int)bz * IP_FAN_CHUNK + la < a_end && lj < beta)
            my_sk = f.key[bz * IP_FAN_CHUNK + la][(size_t)eva.kdig * nmod * n + (size_t)lj * nmod + mi];
    }
    for (int a = bz * IP_FAN_CHUNK; a < a_end; a++) {
        const unsigned dst = perm_src(s2, f.ginv[a], logn);       // where this rotation puts source s2; s2 + 1 goes to dst ^ 1
        const unsigned base = dst & ~1u;
        const bool swap = dst & 1u;
        const u64 *key = f.key[a];
        const u64 cg0 = ((u64)base + 1) * GOLD, cg1 = cg0 + GOLD;
        // every key word of this rotation is requested before the first is used
        ulonglong2 eb[IP_SHARED_MAX_BETA], ea[IP_SHARED_MAX_BETA];
#pragma unroll
        for (int j = 0; j < IP_SHARED_MAX_BETA; j++)
            if (j < beta) {
                const u64 *kb = key + ((size_t)j * nmod + mi) * n + base;
                eb[j].x = __builtin_nontemporal_load(kb), eb[j].y = __builtin_nontemporal_load(kb + 1);
                if (SA) {
                    const u64 *ka = kb + eva.a_off;
                    ea[j].x = __builtin_nontemporal_load(ka), ea[j].y = __builtin_nontemporal_load(ka + 1);
                }
            }
        if (!SA) {
            // attempt 0 of every draw in straight-line code; the rejected ones (a 2^-14 chance under a 50-bit modulus,
            // up to 1/16 under a 60-bit one) are redone in one branch behind them
            const int l0 = (a - (int)bz * IP_FAN_CHUNK) * 8;
            bool rej = false;
#pragma unroll
            for (int j = 0; j < IP_SHARED_MAX_BETA; j++)
                if (j < beta) {
                    const u64 sk_ = ((u64)__builtin_amdgcn_readlane((int)(my_sk >> 32), l0 + j) << 32) |
                                    (unsigned)__builtin_amdgcn_readlane((int)my_sk, l0 + j);
                    ea[j].x = mix64(sk_ + cg0), ea[j].y = mix64(sk_ + cg1);
                    rej |= (ea[j].x >= bound) | (ea[j].y >= bound);
                }
            if (rej) {
#pragma unroll
                for (int j = 0; j < IP_SHARED_MAX_BETA; j++)
                    if (j < beta) {
                        const u64 sk_ = ((u64)__builtin_amdgcn_readlane((int)(my_sk >> 32), l0 + j) << 32) |
                                        (unsigned)__builtin_amdgcn_readlane((int)my_sk, l0 + j);
                        ea[j].x = evk_a_draw(sk_, cg0, base, bound), ea[j].y = evk_a_draw(sk_, cg1, base + 1, bound);
                    }
            }
        }
        u128 a0 = 0, a1 = 0, b0 = 0, b1 = 0;
        if (small) {
            Acc50 A0, A1, B0, B1;
#pragma unroll
            for (int j = 0; j < IP_SHARED_MAX_BETA; j++) {
                if (j < beta) {
                    const u64 dx = swap ? d[j].y : d[j].x, dy = swap ? d[j].x : d[j].y;      // sources of positions base, base + 1
                    const unsigned x0 = (unsigned)dx & LOW25, x1 = (unsigned)(dx >> 25), y0 = (unsigned)dy & LOW25, y1 = (unsigned)(dy >> 25);
                    B0.mac(x0, x1, eb[j].x), B1.mac(y0, y1, eb[j].y);
                    A0.mac(x0, x1, ea[j].x), A1.mac(y0, y1, ea[j].y);
                }
            }
            a0 = A0.total(), a1 = A1.total(), b0 = B0.total(), b1 = B1.total();
        } else {
#pragma unroll
            for (int j = 0; j < IP_SHARED_MAX_BETA; j++) {
                if (j < beta) {
                    const u64 dx = swap ? d[j].y : d[j].x, dy = swap ? d[j].x : d[j].y;
                    b0 += (u128)dx * eb[j].x;
                    b1 += (u128)dy * eb[j].y;
                    a0 += (u128)dx * ea[j].x;
                    a1 += (u128)dy * ea[j].y;
                }
            }
        }
        ulonglong2 r0 = make_ulonglong2(redc(b0, m.q, m.qinv), redc(b1, m.q, m.qinv));
        if (have_c0) r0.x = addmod(r0.x, swap ? cv.y : cv.x, m.q), r0.y = addmod(r0.y, swap ? cv.x : cv.y, m.q);
        const size_t o = (size_t)r * n + base;
        // the rotated ciphertexts are read back much later (by the multiply-accumulate kernel): streamed past the caches
        const u64x2 w0 = {r0.x, r0.y}, w1 = {evk_a_reduce<SA>(a0, m), evk_a_reduce<SA>(a1, m)};
        __builtin_nontemporal_store(w0, reinterpret_cast<u64x2 *>(f.out[a] + o));
        __builtin_nontemporal_store(w1, reinterpret_cast<u64x2 *>(f.out[a] + (size_t)ext * n + o));
    }
}
bool launch_inner_product_fanout(cm_ctx *ctx, const IpFan &f, const u64 *dig, const u64 *c0, bool c0_ext, int beta, int level,
                                 hipStream_t st) {
    if (beta > IP_SHARED_MAX_BETA || f.n < 1 || f.n > IP_FAN_MAX) return false;
    Prof prof_(ctx, CM_K_INNER_PRODUCT, f.n, st);
    const int ext = level + 1 + ctx->K;
    const dim3 grid(ctx->n / (2 * TPB), ext, (f.n + IP_FAN_CHUNK - 1) / IP_FAN_CHUNK);
    if (ctx->evk_stored_a)
        hipLaunchKernelGGL(k_inner_product_fanout<true>, grid, dim3(TPB), 0, st, f, dig, c0, c0_ext ? 1 : 0, ctx->d_modc, beta, ext,
                           level, ctx->L, ctx->nmod, ctx->n, ctx->logn, ctx->d_pmont, evk_a_of(ctx), ctx->d_ubound);
    else
        hipLaunchKernelGGL(k_inner_product_fanout<false>, grid, dim3(TPB), 0, st, f, dig, c0, c0_ext ? 1 : 0, ctx->d_modc, beta, ext,
                           level, ctx->L, ctx->nmod, ctx->n, ctx->logn, ctx->d_pmont, evk_a_of(ctx), ctx->d_ubound);
    return true;
}
// NA keys (rotation amounts) applied to the same nz digit arrays, summed: out[z] = extra[z] + sum_a [ sum_j
// sigma_a(dig_z,j) key_a,j + (sigma_a(c0_z), 0) ].  A lane keeps the words of all NA keys in registers (at most
// IP_MULTI_BETA digits) and writes every output once: against one launch per amount this saves the read-modify-write
// of the running sum, a third of the traffic of the rotation step of an unrolled ladder.
#define IP_MULTI_BETA 6
template <int NA, bool SA>
__global__ __launch_bounds__(TPB) void k_inner_product_multi_key(IpBatch b, IpKeys ks, const ModC *__restrict__ modc, int beta,
                                                                 int ext, int level, int L, int nmod, int n, int logn, EvkA eva,
                                                                 const u64 *__restrict__ ubound) {
    const unsigned i2 = (blockIdx.x * TPB + threadIdx.x) * 2;
    const int r = blockIdx.y;
    const int mi = r <= level ? r : L + 1 + (r - level - 1);
    const ModC m = modc[mi];
    const size_t o = (size_t)r * n + i2;
    const u64 bound = ubound[mi], cg0 = ((u64)i2 + 1) * GOLD, cg1 = cg0 + GOLD;
    ulonglong2 eb[NA][IP_MULTI_BETA], ea[NA][IP_MULTI_BETA];
    unsigned base[NA];
    bool swap[NA];
#pragma unroll
    for (int a = 0; a < NA; a++) {
        const unsigned src = perm_src(i2, ks.g[a], logn);
        base[a] = src & ~1u, swap[a] = src & 1u;
#pragma unroll
        for (int j = 0; j < IP_MULTI_BETA; j++) {
            if (j < beta) {
                const u64 *kb = ks.key[a] + ((size_t)j * nmod + mi) * n + i2;
                eb[a][j].x = __builtin_nontemporal_load(kb), eb[a][j].y = __builtin_nontemporal_load(kb + 1);
                ea[a][j] = evk_a_words<SA>(ks.key[a], eva, nmod, n, j, mi, i2, cg0, cg1, bound);
            }
        }
    }
    for (int z = 0; z < b.nz; z++) {
        const u64 *dig = b.it[z].dig;
        ulonglong2 r0 = make_ulonglong2(0, 0), r1 = make_ulonglong2(0, 0);
        if (b.extra[z]) {
            r0 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + o);
            r1 = *reinterpret_cast<const ulonglong2 *>(b.extra[z] + (size_t)ext * n + o);
        }
#pragma unroll
        for (int a = 0; a < NA; a++) {
            u128 a0 = 0, a1 = 0, b0 = 0, b1 = 0;
#pragma unroll
            for (int j = 0; j < IP_MULTI_BETA; j++) {
                if (j < beta) {
                    ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(dig + ((size_t)j * ext + r) * n + base[a]);
                    const u64 dx = swap[a] ? d.y : d.x, dy = swap[a] ? d.x : d.y;
                    b0 += (u128)dx * eb[a][j].x;
                    b1 += (u128)dy * eb[a][j].y;
                    a0 += (u128)dx * ea[a][j].x;
                    a1 += (u128)dy * ea[a][j].y;
                }
            }
            r0.x = addmod(r0.x, redc(b0, m.q, m.qinv), m.q), r0.y = addmod(r0.y, redc(b1, m.q, m.qinv), m.q);
            r1.x = addmod(r1.x, evk_a_reduce<SA>(a0, m), m.q), r1.y = addmod(r1.y, evk_a_reduce<SA>(a1, m), m.q);
            if (b.it[z].c0) {
                ulonglong2 d = *reinterpret_cast<const ulonglong2 *>(b.it[z].c0 + (size_t)r * n + base[a]);
                r0.x = addmod(r0.x, swap[a] ? d.y : d.x, m.q), r0.y = addmod(r0.y, swap[a] ? d.x : d.y, m.q);
            }
        }
        *reinterpret_cast<ulonglong2 *>(b.out[z] + o) = r0;
        *reinterpret_cast<ulonglong2 *>(b.out[z] + (size_t)ext * n + o) = r1;
    }
}
bool launch_inner_product_multi_key(cm_ctx *ctx, const IpBatch &b, const IpKeys &ks, int na, int beta, int level, hipStream_t st) {
    if (beta > IP_MULTI_BETA || na < 2 || na > IP_MULTI_KEYS) return false;
    const int ext = level + 1 + ctx->K;
    const dim3 grid(ctx->n / (2 * TPB), ext), block(TPB);
    Prof prof_(ctx, CM_K_INNER_PRODUCT, b.nz * na, st);
#define MULTI_KEY_LAUNCH(NA_, SA_)                                                                                          \
    hipLaunchKernelGGL((k_inner_product_multi_key<NA_, SA_>), grid, block, 0, st, b, ks, ctx->d_modc, beta, ext, level, ctx->L, \
                       ctx->nmod, ctx->n, ctx->logn, evk_a_of(ctx), ctx->d_ubound)
    if (na == 2 && ctx->evk_stored_a) MULTI_KEY_LAUNCH(2, true);
    else if (na == 2) MULTI_KEY_LAUNCH(2, false);
    else if (ctx->evk_stored_a) MULTI_KEY_LAUNCH(3, true);
    else MULTI_KEY_LAUNCH(3, false);
#undef MULTI_KEY_LAUNCH
    return true;
}
void launch_inner_product_batch(cm_ctx *ctx, const IpBatch &b, int beta, int level, hipStream_t st) {
    Prof prof_(ctx, CM_K_INNER_PRODUCT, b.nz * b.nsum, st);
    int ext = level + 1 + ctx->K;
    const dim3 grid(ctx->n / (2 * TPB), ext, b.nz);
    if (ctx->evk_stored_a)
        hipLaunchKernelGGL(k_inner_product_batch<true>, grid, dim3(TPB), 0, st, b, ctx->d_modc, beta, ext, level, ctx->L, ctx->nmod,
                           ctx->n, ctx->logn, ctx->d_pmont, evk_a_of(ctx), ctx->d_ubound);
    else
        hipLaunchKernelGGL(k_inner_product_batch<false>, grid, dim3(TPB), 0, st, b, ctx->d_modc, beta, ext, level, ctx->L, ctx->nmod,
                           ctx->n, ctx->logn, ctx->d_pmont, evk_a_of(ctx), ctx->d_ubound);
}
// out[2][ext][n] = (P c0, P c1) on the ciphertext limbs, zero on the special limbs
__global__ void k_raise_by_P(u64 *__restrict__ out, const u64 *__restrict__ in, const ModC *__restrict__ modc,
                             const u64 *__restrict__ pmont, int level, int ext, int n, size_t in_stride, size_t out_stride) {
    int i = blockIdx.x * TPB + threadIdx.x, r = blockIdx.y, c = blockIdx.z & 1;
    in += (blockIdx.z >> 1) * in_stride, out += (blockIdx.z >> 1) * out_stride;      // stacked ciphertexts
    u64 v = 0;
    if (r <= level) {
        const ModC m = modc[r];
        v = redc((u128)in[((size_t)c * (level + 1) + r) * n + i] * pmont[r], m.q, m.qinv);
    }
    out[((size_t)c * ext + r) * n + i] = v;
}
void launch_raise_by_P(cm_ctx *ctx, u64 *out, const u64 *in, int level, hipStream_t st, int count) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, count * 2 * (level + 1 + ctx->K), st);
    int ext = level + 1 + ctx->K;
    hipLaunchKernelGGL(k_raise_by_P, dim3(ctx->n / TPB, ext, 2 * count), dim3(TPB), 0, st, out, in, ctx->d_modc, ctx->d_pmont,
                       level, ext, ctx->n, 2 * (size_t)(level + 1) * ctx->n, 2 * (size_t)ext * ctx->n);
}
void launch_inner_product(cm_ctx *ctx, u64 *u0, u64 *u1, const u64 *dig, const u64 *evk, int beta, int level, u64 g,
                          hipStream_t st, const u64 *c0, const u64 *extra) {
    Prof prof_(ctx, CM_K_INNER_PRODUCT, 1, st);
    int ext = level + 1 + ctx->K;
    if (ctx->evk_stored_a)
        hipLaunchKernelGGL(k_inner_product<true>, dim3(ctx->n / (2 * TPB), ext), dim3(TPB), 0, st, u0, u1, dig, evk, ctx->d_modc,
                           beta, ext, level, ctx->L, ctx->nmod, ctx->n, ctx->logn, (unsigned)g, c0, ctx->d_pmont, extra,
                           evk_a_of(ctx), ctx->d_ubound);
    else
        hipLaunchKernelGGL(k_inner_product<false>, dim3(ctx->n / (2 * TPB), ext), dim3(TPB), 0, st, u0, u1, dig, evk, ctx->d_modc,
                           beta, ext, level, ctx->L, ctx->nmod, ctx->n, ctx->logn, (unsigned)g, c0, ctx->d_pmont, extra,
                           evk_a_of(ctx), ctx->d_ubound);
}

// ---- ModDown tail: out = (u - conv) * P^{-1} (+ addend, optionally through the Galois map) ------------
// batch (blockIdx.z) = component; u rows [ext][n], conv rows [level+1][n], out rows [level+1][n]
__global__ __launch_bounds__(TPB) void k_moddown_finish(u64 *out, const u64 *__restrict__ u, const u64 *__restrict__ conv,
                                 const u64 *__restrict__ pinv, const u64 *__restrict__ addend,
                                 const ModC *__restrict__ modc, int n, int logn, unsigned g, size_t u_stride,
                                 size_t conv_stride, size_t out_stride, int addend_comp_only, const u64 *accum) {
    unsigned i = blockIdx.x * TPB + threadIdx.x;
    int l = blockIdx.y, c = blockIdx.z;
    u64 q = modc[l].q;
    u64 d = submod(u[c * u_stride + (size_t)l * n + i], conv[c * conv_stride + (size_t)l * n + i], q);
    u64 v = mul_shoup(d, pinv[2 * l], pinv[2 * l + 1], q);
    if (addend && c <= addend_comp_only) {
        unsigned s = g ? perm_src(i, g, logn) : i;
        v = addmod(v, addend[c * out_stride + (size_t)l * n + s], q);
    }
    if (accum) v = addmod(v, accum[c * out_stride + (size_t)l * n + i], q);      // out = accum + result
    out[c * out_stride + (size_t)l * n + i] = v;
}
void launch_moddown_finish(cm_ctx *ctx, u64 *out, const u64 *u, const u64 *conv, const u64 *d_pinv, const u64 *addend,
                           int addend_comps, int level, u64 g, const u64 *accum, hipStream_t st, int ncomp) {
    Prof prof_(ctx, CM_K_MODDOWN_FINISH, 1, st);
    int ext = level + 1 + ctx->K;
    size_t n = ctx->n;
    hipLaunchKernelGGL(k_moddown_finish, dim3(ctx->n / TPB, level + 1, ncomp), dim3(TPB), 0, st, out, u, conv, d_pinv,
                       addend, ctx->d_modc, ctx->n, ctx->logn, (unsigned)g, (size_t)ext * n, (size_t)(level + 1) * n,
                       (size_t)(level + 1) * n, addend_comps - 1, accum);
}

// ---- rescale ---------------------------------------------------------------------------------
// last[comp][n]: coefficient-domain last limb in [0, q_l) -> red[comp][l][n] = last mod q_i
__global__ void k_rescale_reduce(u64 *red, const u64 *last, const ModC *modc, int level, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y, c = blockIdx.z;
    const ModC m = modc[l];
    u64 v = last[(size_t)c * n + i];
    red[((size_t)c * level + l) * n + i] = redc((u128)to_mont(v, m), m.q, m.qinv);
}
// out[comp][l][n] = (in[comp][l] - red[comp][l]) * q_level^{-1}; in has level+1 rows per component
// accumulate: out += the result (out holds a running sum of the same shape)
__global__ void k_rescale_finish(u64 *out, const u64 *in, const u64 *red, const u64 *qlinv, const ModC *modc, int level, int n,
                                 int accumulate) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y, c = blockIdx.z;
    u64 q = modc[l].q;
    u64 d = submod(in[((size_t)c * (level + 1) + l) * n + i], red[((size_t)c * level + l) * n + i], q);
    u64 v = mul_shoup(d, qlinv[2 * l], qlinv[2 * l + 1], q);
    const size_t o = ((size_t)c * level + l) * n + i;
    out[o] = accumulate ? addmod(out[o], v, q) : v;
}
void launch_rescale_reduce(cm_ctx *ctx, u64 *red, const u64 *last, int ncomp, int level, hipStream_t st) {
    Prof prof_(ctx, CM_K_RESCALE, ncomp * level, st);
    hipLaunchKernelGGL(k_rescale_reduce, dim3(ctx->n / TPB, level, ncomp), dim3(TPB), 0, st, red, last, ctx->d_modc, level, ctx->n);
}
void launch_rescale_finish(cm_ctx *ctx, u64 *out, const u64 *in, const u64 *red, const u64 *d_qlinv, int ncomp, int level, hipStream_t st,
                           bool accumulate) {
    Prof prof_(ctx, CM_K_RESCALE, ncomp * level, st);
    hipLaunchKernelGGL(k_rescale_finish, dim3(ctx->n / TPB, level, ncomp), dim3(TPB), 0, st, out, in, red, d_qlinv, ctx->d_modc, level, ctx->n,
                       accumulate ? 1 : 0);
}

// ---- counter-based sampling (must reproduce the generator's published definition bit for bit) --------
u64 rng_key(u64 seed, u64 stream) { return mix64(mix64(seed) ^ stream); }
u64 rng_draw(u64 key, u64 ctr) { return mix64(key + (ctr + 1) * GOLD); }

// uniform residues: row l uses stream stream_base | mod_idx[l]
__global__ void k_sample_uniform(u64 *out, const int *mod_idx, const ModC *modc, int n, u64 mseed, u64 stream_base) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    int mi = mod_idx[l];
    u64 q = modc[mi].q;
    u64 key = mix64(mseed ^ (stream_base | (u64)mi));
    // bound = q * floor(2^64 / q): floor(2^64/q) = floor((2^64 - 1)/q) because q is odd > 1
    u64 bound = q * (0xFFFFFFFFFFFFFFFFULL / q);
    u64 att = 0, v;
    do {
        v = mix64(key + (((att << 32) | (u64)i) + 1) * GOLD);
        att++;
    } while (v >= bound);
    out[(size_t)l * n + i] = v % q;
}
void launch_sample_uniform(cm_ctx *ctx, u64 *out, const int *d_mod_idx, int limbs, u64 seed, u64 stream_base, hipStream_t st) {
    hipLaunchKernelGGL(k_sample_uniform, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, d_mod_idx, ctx->d_modc, ctx->n,
                       mix64(seed), stream_base);
}
// one Gaussian integer per coefficient, written as residues to every row
__global__ void k_sample_gauss(u64 *out, const int *mod_idx, const ModC *modc, const u64 *cdt, int limbs, int n, u64 key) {
    int i = blockIdx.x * TPB + threadIdx.x;
    u64 v = mix64(key + ((u64)i + 1) * GOLD), u = v >> 1;
    u64 mag = 0;
    for (int k = 0; k < CM_GAUSS_K; k++) mag += (u >= cdt[k]);
    bool neg = (v & 1) && mag;
    for (int l = 0; l < limbs; l++) {
        u64 q = modc[mod_idx[l]].q;
        out[(size_t)l * n + i] = neg ? q - mag : mag;
    }
}
void launch_sample_gauss(cm_ctx *ctx, u64 *out, const int *d_mod_idx, int limbs, u64 seed, u64 stream, hipStream_t st) {
    hipLaunchKernelGGL(k_sample_gauss, dim3(ctx->n / TPB), dim3(TPB), 0, st, out, d_mod_idx, ctx->d_modc, ctx->d_cdt, limbs,
                       ctx->n, rng_key(seed, stream));
}

// ---- keys and encryption ---------------------------------------------------------------------------
// b = e - a s + fac_l * s_from, then (b, a) stored in multiplier form.  s_mont: secret, evaluation
// domain, multiplier form, rows = all moduli.  s_from = s through the Galois map g (g != 0) or s^2.
__global__ void k_evk_assemble(u64 *b_out, const u64 *a_in, const u64 *e, const u64 *s_mont, const u64 *fac,
                               const ModC *modc, int n, int logn, unsigned g) {
    unsigned i = blockIdx.x * TPB + threadIdx.x;
    int l = blockIdx.y;
    const ModC m = modc[l];
    size_t o = (size_t)l * n + i;
    u64 a = a_in[o];
    u64 b = submod(e[o], redc((u128)a * s_mont[o], m.q, m.qinv), m.q);
    u64 f = fac[l];
    if (f) {
        u64 sf = g ? s_mont[(size_t)l * n + perm_src(i, g, logn)]
                   : redc((u128)s_mont[o] * s_mont[o], m.q, m.qinv);      // s^2 in multiplier form
        b = addmod(b, redc((u128)f * sf, m.q, m.qinv), m.q);
    }
    b_out[o] = to_mont(b, m);
}
void launch_evk_assemble(cm_ctx *ctx, u64 *b_out, const u64 *a_in, const u64 *e, const u64 *s_mont, const u64 *d_fac, u64 g, hipStream_t st) {
    hipLaunchKernelGGL(k_evk_assemble, dim3(ctx->n / TPB, ctx->nmod), dim3(TPB), 0, st, b_out, a_in, e, s_mont, d_fac,
                       ctx->d_modc, ctx->n, ctx->logn, (unsigned)g);
}
// c0 = e - a s + m
__global__ void k_encrypt(u64 *c0, const u64 *a, const u64 *e, const u64 *s_mont, const u64 *pt, const ModC *modc, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[l];
    size_t o = (size_t)l * n + i;
    u64 v = submod(e[o], redc((u128)a[o] * s_mont[o], m.q, m.qinv), m.q);
    c0[o] = addmod(v, pt[o], m.q);
}
void launch_encrypt(cm_ctx *ctx, u64 *c0, const u64 *a, const u64 *e, const u64 *s_mont, const u64 *pt, int limbs, hipStream_t st) {
    hipLaunchKernelGGL(k_encrypt, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, c0, a, e, s_mont, pt, ctx->d_modc, ctx->n);
}
// out = c0 + c1 s (+ c2 s^2) on the first `limbs` limbs; ct rows per component = ct_limbs
__global__ void k_decrypt(u64 *out, const u64 *ct, const u64 *s_mont, const ModC *modc, int ncomp, int ct_limbs, int n) {
    int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const ModC m = modc[l];
    size_t o = (size_t)l * n + i, cs = (size_t)ct_limbs * n;
    u64 s = s_mont[o];
    u64 acc = addmod(ct[o], redc((u128)ct[o + cs] * s, m.q, m.qinv), m.q);
    if (ncomp == 3) {
        u64 s2 = redc((u128)s * s, m.q, m.qinv);
        acc = addmod(acc, redc((u128)ct[o + 2 * cs] * s2, m.q, m.qinv), m.q);
    }
    out[o] = acc;
}
void launch_decrypt(cm_ctx *ctx, u64 *out, const u64 *ct, const u64 *s_mont, int ncomp, int ct_limbs, int limbs, hipStream_t st) {
    hipLaunchKernelGGL(k_decrypt, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, out, ct, s_mont, ctx->d_modc, ncomp, ct_limbs, ctx->n);
}

// ---- packed product: inner_k = sum_j baby_j * p_{j,k} ---------------------------------------------------
// babies: r_i ciphertexts [2][limbs][n] at stride ct_stride; out: r_o ciphertexts at stride
// ct_stride; pts: the r_i*r_o plaintexts in multiplier form, blocked for streaming:
//     word c of chunk ch (64 coefficients) of limb l of plaintext (j,k) at
//     (((l*(n/64) + ch)*r_o + k)*r_i + j)*64 + c
// so that the workgroup that owns (l, ch) reads one contiguous run of r_o*r_i*512 bytes, and the
// wave that owns k one run of r_i*512 bytes.  Limb l has
// modulus index l up to `level`, and the special primes follow when limbs = level + 1 + K (sums
// kept in the extended basis).
// The baby ciphertexts are staged in LDS: a workgroup owns 64 coefficients of
// one limb; its four waves take the k = k0 + wave, k0 + wave + 4, ... and every lane sums over all
// j for its k, so each output is written once and each plaintext word is read once.  Up to 32
// baby ciphertexts per pass (32 KiB of LDS).
#define MAC_CO 64
// the baby ciphertexts are read once per launch, like the plaintexts: non-temporal loads (2 % off the kernel)
#define MAC_LD(ptr) __builtin_nontemporal_load(ptr)
#define MAC_JC 32
#define MAC_KW 4      // giant steps per wave whose sums stay in registers over the passes
#define MAC_G 8       // plaintext words a lane keeps in flight per group (the next group is loaded while one is multiplied; 16 and 32 measured slower)
// Limbs whose modulus is below 2^50 run the products in FP64 (the arithmetic of the transforms'
// butterflies): residues as exact integers in doubles, a modular product
//     h = y a;  l = fma(y, a, -h);  c = rint(y (a / q));  r = fma(-c, q, h) + l        (|r| < q)
// with a / q taken as a * (1 / q), once per plaintext word for both ciphertext components; partial
// sums are renormalised every four terms (|sum| < 4.6 q < 2^53 stays exact).  That is 8.5
// instructions per product against 17 for the 128-bit integer form.  The plaintexts are stored in
// multiplier form (times 2^64), so the finished sum is multiplied by 2^-64 mod q.
// With an even number of baby steps the words of plaintexts (2j', k) and (2j'+1, k) are interleaved
// (word c of the pair at 2c, 2c+1 of a 128-word row), so that a lane reads both with one 16-byte load and a
// wavefront instruction covers 1 KiB of the stream.
__host__ __device__ __forceinline__ size_t mac_pt_index(int n, int r_i, int r_o, int l, int ch, int k, int j, int c) {
    const size_t row = (((size_t)l * (n / MAC_CO) + ch) * r_o + k) * r_i;
    return (r_i & 1) ? (row + j) * MAC_CO + c : (row + (j & ~1)) * MAC_CO + 2 * c + (j & 1);
}
__global__ __launch_bounds__(TPB) void k_vmm_mac_lds(u64 *__restrict__ out, const u64 *__restrict__ babies,
                                                     const u64 *__restrict__ pts, const ModC *__restrict__ modc,
                                                     const FpQ *__restrict__ fpq, int r_i, int r_o, int limbs, int n,
                                                     size_t ct_stride, int k0, int k1, int level, int L) {
    __shared__ u64 sb[MAC_JC * 2 * MAC_CO];
    // the limbs of the special primes (integer products, the slowest workgroups) are dispatched first, not last
    const int nsp = limbs - (level + 1), y = blockIdx.y;
    const int l = y < nsp ? level + 1 + y : y - nsp, ch = blockIdx.x, i0 = ch * MAC_CO;
    const int co = threadIdx.x & (MAC_CO - 1), kq = threadIdx.x >> 6;
    const int mi = l <= level ? l : L + 1 + (l - level - 1);
    const ModC m = modc[mi];
    const FpQ fq = fpq[mi];
    const bool fp = fq.q != 0.0;
    const bool pair = !(r_i & 1);
    const MacFp F{fq.q, fq.qinv};
    const size_t o = (size_t)l * n + i0, cs = (size_t)limbs * n;
    const u64 *pblk = pts + ((size_t)l * (n / MAC_CO) + ch) * r_o * r_i * MAC_CO;
    // up to MAC_KW giant steps per wave keep their running sums in registers across the passes over the baby steps
    // (otherwise every pass after the first re-reads and re-writes the output)
    u64 acc0[MAC_KW], acc1[MAC_KW];
#pragma unroll
    for (int x = 0; x < MAC_KW; x++) acc0[x] = acc1[x] = 0;
    const bool keep = k1 - k0 <= 4 * MAC_KW;
    for (int j0 = 0; j0 < r_i; j0 += MAC_JC) {
        const int jn = r_i - j0 < MAC_JC ? r_i - j0 : MAC_JC;
        __syncthreads();
        {
            // a lane stages word `co` of rows kq, kq + 4, ...: all its loads are issued before the first is used
            constexpr int ROWS = MAC_JC * 2 * MAC_CO / TPB;
            u64 w[ROWS];
#pragma unroll
            for (int it = 0; it < ROWS; it++) {
                const int jc = kq + 4 * it;
                w[it] = jc < 2 * jn ? MAC_LD(babies + (size_t)(j0 + (jc >> 1)) * ct_stride + (jc & 1) * cs + o + co) : 0;
            }
#pragma unroll
            for (int it = 0; it < ROWS; it++) {
                const int jc = kq + 4 * it;
                if (jc < 2 * jn) sb[jc * MAC_CO + co] = fp ? (u64)__double_as_longlong(MacFp::from_u64(w[it])) : w[it];
            }
        }
        __syncthreads();
        // A sum of products is reduced when one more group of 8 could pass q * 2^64 (the bound of
        // REDC): after every group for the 60-bit special primes.
        for (int k = k0 + kq; k < k1; k += 4) {
            const u64 *pk = pblk + ((size_t)k * r_i + j0) * MAC_CO;
            // words of plaintexts j0 + j8 .. j0 + j8 + MAC_G - 1 for this lane's coefficient (zero past the end)
            auto load_group = [&](int j8, u64 (&w)[MAC_G]) {
                if (pair) {
#pragma unroll
                    for (int jj = 0; jj < MAC_G; jj += 2) {
                        u64x2 v = {0, 0};
                        if (j8 + jj < jn) v = __builtin_nontemporal_load(reinterpret_cast<const u64x2 *>(pk + (size_t)(j8 + jj) * MAC_CO) + co);
                        w[jj] = v.x, w[jj + 1] = v.y;
                    }
                } else {
#pragma unroll
                    for (int jj = 0; jj < MAC_G; jj++) w[jj] = j8 + jj < jn ? __builtin_nontemporal_load(pk + (size_t)(j8 + jj) * MAC_CO + co) : 0;
                }
            };
            u64 p[MAC_G], pn[MAC_G];
            load_group(0, p);
            u64 v0, v1;
            if (fp) {
                double s0 = 0.0, s1 = 0.0;
                for (int j8 = 0; j8 < jn; j8 += MAC_G) {
                    // the next group is in flight while this one is multiplied
                    load_group(j8 + MAC_G, pn);
#pragma unroll
                    for (int jj = 0; jj < MAC_G; jj++) {
                        if (j8 + jj < jn) {
                            const double a = MacFp::from_u64(p[jj]), aq = a * F.qinv;
                            s0 += F.mulmod(__longlong_as_double((long long)sb[((j8 + jj) * 2 + 0) * MAC_CO + co]), a, aq);
                            s1 += F.mulmod(__longlong_as_double((long long)sb[((j8 + jj) * 2 + 1) * MAC_CO + co]), a, aq);
                        }
                        if ((jj & 3) == 3) s0 = F.norm(s0), s1 = F.norm(s1);
                    }
#pragma unroll
                    for (int jj = 0; jj < MAC_G; jj++) p[jj] = pn[jj];
                }
                v0 = F.canon(F.mulmod(s0, fq.rinv, fq.rinvq));
                v1 = F.canon(F.mulmod(s1, fq.rinv, fq.rinvq));
            } else {
                v0 = v1 = 0;
                for (int j8 = 0; j8 < jn; j8 += MAC_G) {
                    load_group(j8 + MAC_G, pn);
#pragma unroll
                    for (int h = 0; h < MAC_G; h += 8) {
                        u128 s0 = 0, s1 = 0;
#pragma unroll
                        for (int jj = h; jj < h + 8; jj++) {
                            if (j8 + jj < jn) {
                                s0 += (u128)sb[((j8 + jj) * 2 + 0) * MAC_CO + co] * p[jj];
                                s1 += (u128)sb[((j8 + jj) * 2 + 1) * MAC_CO + co] * p[jj];
                            }
                        }
                        v0 = addmod(v0, redc(s0, m.q, m.qinv), m.q);
                        v1 = addmod(v1, redc(s1, m.q, m.qinv), m.q);
                    }
#pragma unroll
                    for (int jj = 0; jj < MAC_G; jj++) p[jj] = pn[jj];
                }
            }
            u64 *dst = out + (size_t)k * ct_stride + o + co;
            if (keep) {
                // the sums of this wave's giant steps stay in registers over the passes and are written once
                const int ki = (k - k0 - kq) >> 2;
                const bool last = j0 + MAC_JC >= r_i;
#pragma unroll
                for (int x = 0; x < MAC_KW; x++)
                    if (x == ki) {
                        if (j0) v0 = addmod(v0, acc0[x], m.q), v1 = addmod(v1, acc1[x], m.q);
                        acc0[x] = v0, acc1[x] = v1;
                    }
                if (last) dst[0] = v0, dst[cs] = v1;
            } else {
                if (j0) {
                    v0 = addmod(v0, dst[0], m.q);
                    v1 = addmod(v1, dst[cs], m.q);
                }
                dst[0] = v0;
                dst[cs] = v1;
            }
        }
    }
}
void launch_vmm_mac(cm_ctx *ctx, u64 *out, const u64 *babies, const u64 *pts, int r_i, int r_o, int limbs, int level,
                    size_t ct_stride, int k0, int k1, hipStream_t st) {
    Prof prof_(ctx, CM_K_VMM_MAC, r_i * (k1 - k0), st);
    hipLaunchKernelGGL(k_vmm_mac_lds, dim3(ctx->n / MAC_CO, limbs), dim3(TPB), 0, st, out, babies, pts, ctx->d_modc,
                       ctx->d_fpq, r_i, r_o, limbs, ctx->n, ct_stride, k0, k1, level, ctx->L);
}
// ---- masks before the shared rotations of query-times-K --------------------------------------------------
// A[k] = sum_{c < nk} T[c] * M[(c + k) mod E] for k < shared: T the nk key-ciphertext sums [2][limbs][n] (stacked),
// M the E slot rotations of the copy mask [E][limbs][n] (multiplier form), A stacked like T.  For one coefficient
// this is a correlation of the vector over c with the vector over the copies, so a lane that owns KO consecutive
// outputs k needs ONE new mask word per c: rows (c + k0) .. (c + k0 + KO - 1) slide by one.  A workgroup owns 64
// coefficients of one limb and stages CIRC_CC ciphertexts at a time in LDS (32 KiB); its four waves take KO outputs
// each.  Limbs below 2^50 multiply in FP64 (MacFp), the others in 128-bit integer sums reduced every 8 terms.
#define CIRC_CC 32
template <int KO>
__global__ __launch_bounds__(TPB) void k_mask_circulant(u64 *__restrict__ A, const u64 *__restrict__ T, const u64 *__restrict__ M,
                                                        const ModC *__restrict__ modc, const FpQ *__restrict__ fpq, int nk, int E,
                                                        int shared, int limbs, int n) {
    __shared__ u64 sb[CIRC_CC * 2 * MAC_CO];
    const int l = blockIdx.y, i0 = blockIdx.x * MAC_CO;
    const int co = threadIdx.x & (MAC_CO - 1), w = threadIdx.x >> 6;
    const int kb = (blockIdx.z * 4 + w) * KO;
    const bool active = kb < shared;
    const ModC m = modc[l];
    const FpQ fq = fpq[l];
    const bool fp = fq.q != 0.0;
    const MacFp F{fq.q, fq.qinv};
    const size_t cs = (size_t)limbs * n, ctw = 2 * cs, o = (size_t)l * n + i0;
    double s[KO][2];
    u64 v[KO][2];
#pragma unroll
    for (int t = 0; t < KO; t++) s[t][0] = s[t][1] = 0.0, v[t][0] = v[t][1] = 0;
    for (int c0 = 0; c0 < nk; c0 += CIRC_CC) {
        const int cn = nk - c0 < CIRC_CC ? nk - c0 : CIRC_CC;
        __syncthreads();
        {
            constexpr int ROWS = CIRC_CC * 2 * MAC_CO / TPB;      // all loads of a lane in flight before the first is used
            u64 x[ROWS];
#pragma unroll
            for (int it = 0; it < ROWS; it++) {
                const int jc = w + 4 * it;
                x[it] = jc < 2 * cn ? T[(size_t)(c0 + (jc >> 1)) * ctw + (jc & 1) * cs + o + co] : 0;
            }
#pragma unroll
            for (int it = 0; it < ROWS; it++) {
                const int jc = w + 4 * it;
                if (jc < 2 * cn) sb[jc * MAC_CO + co] = fp ? (u64)__double_as_longlong(MacFp::from_u64(x[it])) : x[it];
            }
        }
        __syncthreads();
        if (!active) continue;
        for (int c8 = 0; c8 < cn; c8 += 8) {
            u64 wv[KO + 7];
#pragma unroll
            for (int x = 0; x < KO + 7; x++)
                wv[x] = M[((size_t)((c0 + c8 + kb + x) & (E - 1)) * limbs + l) * n + i0 + co];     // E is a power of two
            if (fp) {
                double wa[KO + 7], waq[KO + 7];
#pragma unroll
                for (int x = 0; x < KO + 7; x++) wa[x] = MacFp::from_u64(wv[x]), waq[x] = wa[x] * F.qinv;
#pragma unroll
                for (int cc = 0; cc < 8; cc++) {
                    if (c8 + cc < cn) {
                        const double y0 = __longlong_as_double((long long)sb[((c8 + cc) * 2 + 0) * MAC_CO + co]);
                        const double y1 = __longlong_as_double((long long)sb[((c8 + cc) * 2 + 1) * MAC_CO + co]);
#pragma unroll
                        for (int t = 0; t < KO; t++) {
                            s[t][0] += F.mulmod(y0, wa[cc + t], waq[cc + t]);
                            s[t][1] += F.mulmod(y1, wa[cc + t], waq[cc + t]);
                        }
                    }
                    if ((cc & 3) == 3) {
#pragma unroll
                        for (int t = 0; t < KO; t++) s[t][0] = F.norm(s[t][0]), s[t][1] = F.norm(s[t][1]);
                    }
                }
            } else {
                u128 a[KO][2];
#pragma unroll
                for (int t = 0; t < KO; t++) a[t][0] = a[t][1] = 0;
#pragma unroll
                for (int cc = 0; cc < 8; cc++) {
                    if (c8 + cc < cn) {
                        const u64 y0 = sb[((c8 + cc) * 2 + 0) * MAC_CO + co], y1 = sb[((c8 + cc) * 2 + 1) * MAC_CO + co];
#pragma unroll
                        for (int t = 0; t < KO; t++) a[t][0] += (u128)y0 * wv[cc + t], a[t][1] += (u128)y1 * wv[cc + t];
                    }
                }
#pragma unroll
                for (int t = 0; t < KO; t++) {
                    v[t][0] = addmod(v[t][0], redc(a[t][0], m.q, m.qinv), m.q);
                    v[t][1] = addmod(v[t][1], redc(a[t][1], m.q, m.qinv), m.q);
                }
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int t = 0; t < KO; t++) {
        if (kb + t < shared) {
            u64 *dst = A + (size_t)(kb + t) * ctw + o + co;
            dst[0] = fp ? F.canon(F.mulmod(s[t][0], fq.rinv, fq.rinvq)) : v[t][0];
            dst[cs] = fp ? F.canon(F.mulmod(s[t][1], fq.rinv, fq.rinvq)) : v[t][1];
        }
    }
}
void launch_mask_circulant(cm_ctx *ctx, u64 *A, const u64 *T, const u64 *M, int nk, int E, int shared, int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, (double)nk * shared * 2 * limbs, st);
    const int ko = shared >= 8 ? 8 : shared >= 4 ? 4 : 2;
    const dim3 grid(ctx->n / MAC_CO, limbs, (shared + 4 * ko - 1) / (4 * ko)), block(TPB);
    if (ko == 8)
        hipLaunchKernelGGL(k_mask_circulant<8>, grid, block, 0, st, A, T, M, ctx->d_modc, ctx->d_fpq, nk, E, shared, limbs, ctx->n);
    else if (ko == 4)
        hipLaunchKernelGGL(k_mask_circulant<4>, grid, block, 0, st, A, T, M, ctx->d_modc, ctx->d_fpq, nk, E, shared, limbs, ctx->n);
    else
        hipLaunchKernelGGL(k_mask_circulant<2>, grid, block, 0, st, A, T, M, ctx->d_modc, ctx->d_fpq, nk, E, shared, limbs, ctx->n);
}
// The same sums through a length-E transform along the copy index: for one coefficient A[k] = sum_c t[c] m[(c + k) mod E]
// is a cyclic correlation, so with t'[c] = t[(-c) mod E] and F the length-E number-theoretic transform (E divides
// q - 1), A = F^-1( F(m) . F(t') ): E (log2 E + 1) products per coefficient instead of nk * shared, exact like the direct sum.
// MODE 0 (set-up): rows M[E][limbs][n] -> Mhat = F(m) / E, kept in the order the forward pass leaves (bit-reversed);
// MODE 1: T[nk] stacked ciphertexts -> A[shared].  A workgroup owns CO coefficients of one limb and one component and
// keeps the E x CO words in LDS; the forward pass is decimation in frequency, the inverse one decimation in time, so
// no reordering is needed.  tw[limbs][2][E/2][2]: omega^e and omega^-e with their companions; einv[limbs]: E^-1 in
// multiplier form.
template <int MODE>
__global__ __launch_bounds__(TPB) void k_mask_ntt(u64 *__restrict__ out, const u64 *__restrict__ in, const u64 *__restrict__ Mhat,
                                                  const u64 *__restrict__ tw, const u64 *__restrict__ einv,
                                                  const ModC *__restrict__ modc, int nk, int E, int logE, int shared, int limbs,
                                                  int n, int logCO) {
    extern __shared__ u64 X[];
    const int CO = 1 << logCO, l = blockIdx.y, comp = blockIdx.z, i0 = blockIdx.x * CO;
    const ModC m = modc[l];
    const u64 q = m.q;
    const size_t cs = (size_t)limbs * n, ctw = 2 * cs, o = (size_t)l * n + i0;
    for (int e = threadIdx.x; e < E * CO; e += TPB) {
        const int c = e >> logCO, co = e & (CO - 1);
        if (MODE == 1) X[(((E - c) & (E - 1)) << logCO) + co] = c < nk ? in[(size_t)c * ctw + comp * cs + o + co] : 0;
        else X[e] = in[(size_t)c * cs + o + co];
    }
    __syncthreads();
    const u64 *twf = tw + (size_t)l * 2 * E, *twi = twf + E;
    for (int lg = logE - 1; lg >= 0; lg--) {                       // half-length 2^lg, twiddle step 2^(logE - 1 - lg)
        const int len = 1 << lg, sh = logE - 1 - lg;
        for (int id = threadIdx.x; id < (E / 2) * CO; id += TPB) {
            const int bf = id >> logCO, co = id & (CO - 1), j = bf & (len - 1);
            const int a = ((((bf >> lg) << (lg + 1)) + j) << logCO) + co, b = a + (len << logCO);
            const u64 u = X[a], v = X[b];
            X[a] = addmod(u, v, q);
            const int e = j << sh;
            X[b] = mul_shoup(submod(u, v, q), twf[2 * e], twf[2 * e + 1], q);
        }
        __syncthreads();
    }
    if (MODE == 0) {
        const u64 s = einv[l];
        for (int e = threadIdx.x; e < E * CO; e += TPB)
            out[(size_t)(e >> logCO) * cs + o + (e & (CO - 1))] = redc((u128)X[e] * s, q, m.qinv);
        return;
    }
    for (int e = threadIdx.x; e < E * CO; e += TPB)
        X[e] = redc((u128)X[e] * Mhat[(size_t)(e >> logCO) * cs + o + (e & (CO - 1))], q, m.qinv);
    __syncthreads();
    for (int lg = 0; lg < logE; lg++) {
        const int len = 1 << lg, sh = logE - 1 - lg;
        for (int id = threadIdx.x; id < (E / 2) * CO; id += TPB) {
            const int bf = id >> logCO, co = id & (CO - 1), j = bf & (len - 1);
            const int a = ((((bf >> lg) << (lg + 1)) + j) << logCO) + co, b = a + (len << logCO);
            const int e = j << sh;
            const u64 u = X[a], v = mul_shoup(X[b], twi[2 * e], twi[2 * e + 1], q);
            X[a] = addmod(u, v, q);
            X[b] = submod(u, v, q);
        }
        __syncthreads();
    }
    for (int e = threadIdx.x; e < shared * CO; e += TPB)
        out[(size_t)(e >> logCO) * ctw + comp * cs + o + (e & (CO - 1))] = X[e];
}
// CO = min(64, 4096 / E) coefficients per workgroup (32 KiB of LDS at most); 8 <= E <= 512
static int mask_ntt_log_co(int E) {
    int lg = 6;
    while ((E << lg) > 4096) lg--;
    return lg;
}
bool mask_ntt_supported(int E) { return E >= 8 && E <= 512 && (E & (E - 1)) == 0; }
void launch_mask_ntt_setup(cm_ctx *ctx, u64 *Mhat, const u64 *M, const u64 *tw, const u64 *einv, int E, int limbs, hipStream_t st) {
    int logE = 0;
    while ((1 << logE) < E) logE++;
    const int lg = mask_ntt_log_co(E);
    hipLaunchKernelGGL(k_mask_ntt<0>, dim3(ctx->n >> lg, limbs, 1), dim3(TPB), ((size_t)E << lg) * 8, st, Mhat, M, nullptr, tw, einv,
                       ctx->d_modc, E, E, logE, E, limbs, ctx->n, lg);
}
void launch_mask_ntt(cm_ctx *ctx, u64 *A, const u64 *T, const u64 *Mhat, const u64 *tw, const u64 *einv, int nk, int E, int shared,
                     int limbs, hipStream_t st) {
    Prof prof_(ctx, CM_K_ELEMENTWISE, (double)E * 2 * limbs, st);
    int logE = 0;
    while ((1 << logE) < E) logE++;
    const int lg = mask_ntt_log_co(E);
    hipLaunchKernelGGL(k_mask_ntt<1>, dim3(ctx->n >> lg, limbs, 2), dim3(TPB), ((size_t)E << lg) * 8, st, A, T, Mhat, tw, einv,
                       ctx->d_modc, nk, E, logE, shared, limbs, ctx->n, lg);
}
// plaintext (j,k) between its plain form src[limbs][n] and its place in the blocked array
__global__ void k_pt_block(u64 *blocked, u64 *plain, int n, int r_i, int r_o, int j, int k, int to_blocked) {
    const int i = blockIdx.x * TPB + threadIdx.x, l = blockIdx.y;
    const size_t b = mac_pt_index(n, r_i, r_o, l, i / MAC_CO, k, j, i % MAC_CO);
    const size_t p = (size_t)l * n + i;
    if (to_blocked) blocked[b] = plain[p];
    else plain[p] = blocked[b];
}
void launch_pt_block(cm_ctx *ctx, u64 *blocked, u64 *plain, int limbs, int r_i, int r_o, int j, int k, bool to_blocked,
                     hipStream_t st) {
    hipLaunchKernelGGL(k_pt_block, dim3(ctx->n / TPB, limbs), dim3(TPB), 0, st, blocked, plain, ctx->n, r_i, r_o, j, k,
                       to_blocked ? 1 : 0);
}
