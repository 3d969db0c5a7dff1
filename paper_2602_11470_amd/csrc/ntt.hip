// Batched negacyclic NTT / inverse NTT over RNS limbs for gfx950.
//
// Transform: a(X) in Z_q[X]/(X^n+1)  ->  values a(psi^(2 brev(i)+1)) at position i (bit-reversed
// evaluation order), the merged-twiddle Cooley-Tukey / Gentleman-Sande pair with Harvey's lazy
// butterflies (operands kept below 4q forward, 2q inverse; Shoup twiddles).
//
// Decomposition for the 64-wide machine: n = 256 * n2.  A workgroup of 256 lanes owns 4096
// words; every lane keeps 16 of them in registers and runs four butterfly stages there
// (radix 16), then the workgroup transposes through LDS and runs four more.
//   column kernel : stages 0..7, a tile of 256 rows x 16 adjacent columns (rows n2 apart)
//   row kernel    : the remaining log2(n2) stages on contiguous blocks of n2 words
// so a limb makes two round trips to HBM for n = 65536 (and for n = 4096).
#include "kernels.h"

#define NTT_THREADS 256

// ---- butterflies ---------------------------------------------------------------------------
__device__ __forceinline__ void ct_bfly(u64 &X, u64 &Y, u64 w, u64 wp, u64 q, u64 q2) {
    u64 x = X >= q2 ? X - q2 : X;
    u64 t = mul_shoup_lazy(Y, w, wp, q);
    X = x + t;
    Y = x - t + q2;
}
__device__ __forceinline__ void gs_bfly(u64 &X, u64 &Y, u64 w, u64 wp, u64 q, u64 q2) {
    u64 s = X + Y;
    u64 d = X - Y + q2;
    X = s >= q2 ? s - q2 : s;
    Y = mul_shoup_lazy(d, w, wp, q);
}

// Four forward stages on 16 register values whose index k is the local position inside one
// butterfly block of the first of these stages; base0 = 2^s0 + (block index at stage s0).
__device__ __forceinline__ void radix16_fwd(u64 (&v)[16], const u64 *__restrict__ tw,
                                            const u64 *__restrict__ twp, u64 q, u64 base0) {
    const u64 q2 = 2 * q;
#pragma unroll
    for (int a = 0; a < 4; a++) {
        const int half = 8 >> a;
#pragma unroll
        for (int g = 0; g < (1 << a); g++) {
            u64 idx = (base0 << a) + g;
            u64 w = tw[idx], wp = twp[idx];
#pragma unroll
            for (int j = 0; j < half; j++) {
                int k = g * 2 * half + j;
                ct_bfly(v[k], v[k + half], w, wp, q, q2);
            }
        }
    }
}
// The inverse of the above (stages in the opposite order).  Values in and out below 2q.
__device__ __forceinline__ void radix16_inv(u64 (&v)[16], const u64 *__restrict__ tw,
                                            const u64 *__restrict__ twp, u64 q, u64 base0) {
    const u64 q2 = 2 * q;
#pragma unroll
    for (int a = 3; a >= 0; a--) {
        const int half = 8 >> a;
#pragma unroll
        for (int g = 0; g < (1 << a); g++) {
            u64 idx = (base0 << a) + g;
            u64 w = tw[idx], wp = twp[idx];
#pragma unroll
            for (int j = 0; j < half; j++) {
                int k = g * 2 * half + j;
                gs_bfly(v[k], v[k + half], w, wp, q, q2);
            }
        }
    }
}

// LDS index with one pad word per 16 so that lanes reading words 16 apart hit distinct banks
__device__ __forceinline__ int pad(int e) { return e + (e >> 4); }
#define LDS_WORDS (4096 + 256)

// ---- column kernels: stages 0..7 --------------------------------------------------------------
// grid.x = limbs * (n2/16); tile = rows 0..255 of 16 adjacent columns.
__global__ __launch_bounds__(NTT_THREADS) void ntt_cols_fwd(u64 *__restrict__ data,
                                                           const u64 *__restrict__ src,
                                                           const int *__restrict__ src_rows,
                                                           const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                           const ModC *__restrict__ modc,
                                                           const u64 *__restrict__ tw_all,
                                                           const u64 *__restrict__ twp_all, int n,
                                                           int n2) {
    __shared__ u64 lds[LDS_WORDS];
    const int tiles = n2 >> 4;
    const int limb = blockIdx.x / tiles, c0 = (blockIdx.x % tiles) << 4;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + c0;
    const u64 *ps = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n + c0 : p;
    const int c = threadIdx.x & 15, sub = threadIdx.x >> 4;
    u64 v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ps[(size_t)(sub + 16 * k) * n2 + c];
    radix16_fwd(v, tw, twp, q, 1);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad((sub + 16 * k) * 16 + c)] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = lds[pad((16 * sub + k) * 16 + c)];
    radix16_fwd(v, tw, twp, q, 16 + sub);
#pragma unroll
    for (int k = 0; k < 16; k++) p[(size_t)(16 * sub + k) * n2 + c] = v[k];   // below 4q
}

__global__ __launch_bounds__(NTT_THREADS) void ntt_cols_inv(u64 *__restrict__ data,
                                                           const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                           const ModC *__restrict__ modc,
                                                           const u64 *__restrict__ tw_all,
                                                           const u64 *__restrict__ twp_all,
                                                           const u64 *__restrict__ ninv,
                                                           const u64 *__restrict__ ninvp, int n,
                                                           int n2) {
    __shared__ u64 lds[LDS_WORDS];
    const int tiles = n2 >> 4;
    const int limb = blockIdx.x / tiles, c0 = (blockIdx.x % tiles) << 4;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + c0;
    const int c = threadIdx.x & 15, sub = threadIdx.x >> 4;
    u64 v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = p[(size_t)(16 * sub + k) * n2 + c];   // below 2q
    radix16_inv(v, tw, twp, q, 16 + sub);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad((16 * sub + k) * 16 + c)] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = lds[pad((sub + 16 * k) * 16 + c)];
    radix16_inv(v, tw, twp, q, 1);
    const u64 ni = ninv[mi], nip = ninvp[mi];
#pragma unroll
    for (int k = 0; k < 16; k++) p[(size_t)(sub + 16 * k) * n2 + c] = mul_shoup(v[k], ni, nip, q);
}

// ---- row kernels: stages 8.. on contiguous blocks of n2 words ------------------------------------
// n2 = 256: grid.x = limbs * n/4096, a workgroup owns 16 blocks.
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows256_fwd(u64 *__restrict__ data,
                                                              const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                              const ModC *__restrict__ modc,
                                                              const u64 *__restrict__ tw_all,
                                                              const u64 *__restrict__ twp_all,
                                                              int n) {
    __shared__ u64 lds[LDS_WORDS];
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + (size_t)chunk * 4096;
    const int sub = threadIdx.x & 15, blk = threadIdx.x >> 4;
    const u64 B = (u64)chunk * 16 + blk;
    u64 v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        u64 x = p[blk * 256 + sub + 16 * k];       // below 4q from the column kernel
        v[k] = x;
    }
    radix16_fwd(v, tw, twp, q, 256 + B);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad(blk * 256 + sub + 16 * k)] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = lds[pad(blk * 256 + 16 * sub + k)];
    radix16_fwd(v, tw, twp, q, 4096 + B * 16 + sub);
    const u64 q2 = 2 * q;
#pragma unroll
    for (int k = 0; k < 16; k++) {
        u64 x = v[k];
        x = x >= q2 ? x - q2 : x;
        v[k] = x >= q ? x - q : x;
    }
    // lane owns 16 contiguous words: store as 8 x 16 bytes
    ulonglong2 *o = reinterpret_cast<ulonglong2 *>(p + blk * 256 + 16 * sub);
#pragma unroll
    for (int k = 0; k < 8; k++) o[k] = make_ulonglong2(v[2 * k], v[2 * k + 1]);
}

__global__ __launch_bounds__(NTT_THREADS) void ntt_rows256_inv(u64 *__restrict__ data,
                                                              const u64 *__restrict__ src,
                                                              const int *__restrict__ src_rows,
                                                              const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                              const ModC *__restrict__ modc,
                                                              const u64 *__restrict__ tw_all,
                                                              const u64 *__restrict__ twp_all,
                                                              int n) {
    __shared__ u64 lds[LDS_WORDS];
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + (size_t)chunk * 4096;
    const int sub = threadIdx.x & 15, blk = threadIdx.x >> 4;
    const u64 B = (u64)chunk * 16 + blk;
    u64 v[16];
    const u64 *ps = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n + (size_t)chunk * 4096 : p;
    const ulonglong2 *in = reinterpret_cast<const ulonglong2 *>(ps + blk * 256 + 16 * sub);
#pragma unroll
    for (int k = 0; k < 8; k++) {
        ulonglong2 x = in[k];
        v[2 * k] = x.x;
        v[2 * k + 1] = x.y;
    }
    radix16_inv(v, tw, twp, q, 4096 + B * 16 + sub);
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad(blk * 256 + 16 * sub + k)] = v[k];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = lds[pad(blk * 256 + sub + 16 * k)];
    radix16_inv(v, tw, twp, q, 256 + B);
#pragma unroll
    for (int k = 0; k < 16; k++) p[blk * 256 + sub + 16 * k] = v[k];          // below 2q
}

// n2 = 16: every lane owns one block of 16 contiguous words.  grid.x = limbs * n/4096.
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows16_fwd(u64 *__restrict__ data,
                                                             const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                             const ModC *__restrict__ modc,
                                                             const u64 *__restrict__ tw_all,
                                                             const u64 *__restrict__ twp_all,
                                                             int n) {
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q, q2 = 2 * q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    const u64 B = (u64)chunk * 256 + threadIdx.x;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + B * 16;
    u64 v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = p[k];
    radix16_fwd(v, tw, twp, q, 256 + B);
#pragma unroll
    for (int k = 0; k < 16; k++) {
        u64 x = v[k];
        x = x >= q2 ? x - q2 : x;
        p[k] = x >= q ? x - q : x;
    }
}
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows16_inv(u64 *__restrict__ data,
                                                             const u64 *__restrict__ src,
                                                             const int *__restrict__ src_rows,
                                                             const int *__restrict__ rows,
        const int *__restrict__ mod_idx,
                                                             const ModC *__restrict__ modc,
                                                             const u64 *__restrict__ tw_all,
                                                             const u64 *__restrict__ twp_all,
                                                             int n) {
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 q = modc[mi].q;
    const u64 *tw = tw_all + (size_t)mi * n, *twp = twp_all + (size_t)mi * n;
    const u64 B = (u64)chunk * 256 + threadIdx.x;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + B * 16;
    const u64 *ps = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n + B * 16 : p;
    u64 v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ps[k];
    radix16_inv(v, tw, twp, q, 256 + B);
#pragma unroll
    for (int k = 0; k < 16; k++) p[k] = v[k];
}

// data rows d_rows[i] (or i) are transformed in place; with src != nullptr the first pass reads row
// src_rows[i] (or i) of src instead, so the transform is out of place and src is left untouched.
void launch_ntt_src(cm_ctx *ctx, u64 *data, const int *d_rows, const u64 *src, const int *d_src_rows,
                    const int *d_mod_idx, int limbs, bool inverse, hipStream_t st) {
    if (limbs <= 0) return;
    Prof prof_(ctx, inverse ? CM_K_NTT_INV : CM_K_NTT_FWD, limbs, st);
    const int n = ctx->n, n2 = n >> 8;
    dim3 grid((unsigned)limbs * (n >> 12)), block(NTT_THREADS);
    if (!inverse) {
        hipLaunchKernelGGL(ntt_cols_fwd, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx, ctx->d_modc,
                           ctx->d_tw, ctx->d_twp, n, n2);
        if (n2 == 256)
            hipLaunchKernelGGL(ntt_rows256_fwd, grid, block, 0, st, data, d_rows, d_mod_idx, ctx->d_modc,
                               ctx->d_tw, ctx->d_twp, n);
        else
            hipLaunchKernelGGL(ntt_rows16_fwd, grid, block, 0, st, data, d_rows, d_mod_idx, ctx->d_modc,
                               ctx->d_tw, ctx->d_twp, n);
    } else {
        if (n2 == 256)
            hipLaunchKernelGGL(ntt_rows256_inv, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx,
                               ctx->d_modc, ctx->d_itw, ctx->d_itwp, n);
        else
            hipLaunchKernelGGL(ntt_rows16_inv, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx,
                               ctx->d_modc, ctx->d_itw, ctx->d_itwp, n);
        hipLaunchKernelGGL(ntt_cols_inv, grid, block, 0, st, data, d_rows, d_mod_idx, ctx->d_modc,
                           ctx->d_itw, ctx->d_itwp, ctx->d_ninv, ctx->d_ninvp, n, n2);
    }
}
void launch_ntt_rows(cm_ctx *ctx, u64 *data, const int *d_rows, const int *d_mod_idx, int limbs,
                     bool inverse, hipStream_t st) {
    launch_ntt_src(ctx, data, d_rows, nullptr, nullptr, d_mod_idx, limbs, inverse, st);
}

void launch_ntt(cm_ctx *ctx, u64 *data, const int *d_mod_idx, int limbs, bool inverse,
                hipStream_t st) {
    launch_ntt_rows(ctx, data, nullptr, d_mod_idx, limbs, inverse, st);
}

void launch_ntt_range(cm_ctx *ctx, u64 *data, int first_mod, int limbs, bool inverse,
                      hipStream_t st) {
    launch_ntt(ctx, data, iota_idx(ctx) + first_mod, limbs, inverse, st);
}
