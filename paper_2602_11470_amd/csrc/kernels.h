// Launchers of the kernels in kernels.hip.  All pointers are device pointers unless named h_*.
#pragma once
#include "common.h"

void launch_set_idx(int *d_dst, const int *h_src, int count, hipStream_t st);
void launch_reduce_i64(cm_ctx *ctx, u64 *out, const long long *d_coeffs, const int *d_mod_idx, int limbs, hipStream_t st);
void launch_to_mont(cm_ctx *ctx, u64 *data, const int *d_mod_idx, int limbs, hipStream_t st);
void launch_from_mont(cm_ctx *ctx, u64 *out, const u64 *in, const int *d_mod_idx, int limbs, hipStream_t st);
void launch_add(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int ncomp, int limbs, hipStream_t st);
void launch_mul_pt(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *pt_mont, int ncomp, int limbs, hipStream_t st);
// out[z][2][limbs][n] = src[z] * (pt rotated by the Galois element g[z]) for z < cnt <= CM_KS_BATCH
struct MulPtBatch {
    const u64 *src[CM_KS_BATCH];
    unsigned g[CM_KS_BATCH];
};
void launch_mul_pt_rot_batch(cm_ctx *ctx, u64 *out, const MulPtBatch &b, int cnt, const u64 *pt_mont, int limbs, hipStream_t st);
// the same products on the last of the `limbs` limbs only: out[z][2][n]
void launch_mul_pt_rot_last(cm_ctx *ctx, u64 *out, const MulPtBatch &b, int cnt, const u64 *pt_mont, int limbs, hipStream_t st);
// acc[2][limbs][n] (+)= sum_{z<cnt} src[z] * (pt rotated by b.g[z]), src[z] = src + z*2*limbs*n (b.src unused)
void launch_mac_pt_rot_batch(cm_ctx *ctx, u64 *acc, const u64 *src, const MulPtBatch &b, int cnt, const u64 *pt_mont,
                             int limbs, int accumulate, hipStream_t st);
void launch_mac_pt(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *pt_mont, int ncomp, int limbs, int accumulate, hipStream_t st);
void launch_tensor(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int limbs, int accumulate, hipStream_t st);
// out[z][3][limbs][n] = a (x) b[z], b[z] = b + z*2*limbs*n, z < cnt
// out[z][3][limbs][n] = sum_{j < cnt} a[j] (x) b[z*cnt + j] for z < groups (a, b stacked ciphertexts [2][limbs][n])
// b[z*group_stride + j*term_stride] is term j of group z (0, 0 = groups of cnt consecutive ciphertexts)
void launch_tensor_sum(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int cnt, int groups, int limbs, hipStream_t st,
                       int group_stride = 0, int term_stride = 0);
void launch_tensor_batch(cm_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int cnt, int limbs, hipStream_t st);
void launch_automorphism(cm_ctx *ctx, u64 *out, const u64 *in, int rows, u64 g, hipStream_t st);
// A[k][2][limbs][n] = sum_{c < nk} T[c] * M[(c + k) mod E], k < shared (2 <= shared <= E, powers of two); T, A stacked
// ciphertexts, M[E][limbs][n] in multiplier form; limbs use modulus indices 0 .. limbs-1
void launch_mask_circulant(cm_ctx *ctx, u64 *A, const u64 *T, const u64 *M, int nk, int E, int shared, int limbs, hipStream_t st);
// the same sums through a length-E transform along the copy index (8 <= E <= 512): Mhat[E][limbs][n] from M once
// (set-up), then A from T; tw[limbs][2][E/2][2] = omega^e, omega^-e with companions, einv[limbs] = E^-1 in multiplier form
bool mask_ntt_supported(int E);
void launch_mask_ntt_setup(cm_ctx *ctx, u64 *Mhat, const u64 *M, const u64 *tw, const u64 *einv, int E, int limbs, hipStream_t st);
void launch_mask_ntt(cm_ctx *ctx, u64 *A, const u64 *T, const u64 *Mhat, const u64 *tw, const u64 *einv, int nk, int E, int shared,
                     int limbs, hipStream_t st);
// batch item z: table (z % tab_period)*tab_step (tab_period 0 = batch), input (z / in_group)*in_stride, output z*out_stride
void launch_base_conv(cm_ctx *ctx, const ConvDev *d_tabs, int batch, int tab_step, int max_nt, u64 *out, const u64 *in,
                      size_t in_stride, size_t out_stride, const u64 *own_src, u64 own_g, hipStream_t st,
                      int tab_period = 0, int in_group = 1, size_t own_stride = 0);
// (u0, u1)[ext][n] = sum_j perm_g(dig_j) * evk_j  [+ P * perm_g(c0) on the ciphertext limbs of u0]  [+ extra[2][ext][n]]
void launch_inner_product(cm_ctx *ctx, u64 *u0, u64 *u1, const u64 *dig, const u64 *evk, int beta, int level, u64 g,
                          hipStream_t st, const u64 *c0 = nullptr, const u64 *extra = nullptr);
// Up to IP_MAX_ITEMS inner products in one launch.  Output z < nz (out[z] = [2][ext][n]) is
// extra[z] (nullable, may be out[z] itself) + the sum of items z*nsum .. z*nsum + nsum - 1, each
// sum_j perm_g(dig_j) * key_j [+ P * perm_g(c0) on the ciphertext limbs of the first component].
#define IP_MAX_ITEMS 32
struct IpItem {
    const u64 *dig = nullptr, *key = nullptr, *c0 = nullptr;
    unsigned g = 0;
    unsigned c0_ext = 0;      // c0 is already in the extended basis ([ext][n], all limbs): added as it is, no factor P
};
struct IpBatch {
    int nz = 0, nsum = 1;
    IpItem it[IP_MAX_ITEMS];
    u64 *out[IP_MAX_ITEMS] = {};
    const u64 *extra[IP_MAX_ITEMS] = {};      // nullable; the kernels test it, so it must never be left unset
};
void launch_inner_product_batch(cm_ctx *ctx, const IpBatch &b, int beta, int level, hipStream_t st);
// na = 2 or 3 keys (Galois elements g[a] != 0) applied to the nz digit arrays b.it[z].dig and summed into out[z] together with
// extra[z] and, per key, the first component b.it[z].c0 (extended basis) through that key's Galois map.  Returns false
// (nothing launched) if the lane cannot hold the keys: more than 6 digits.
// Up to IP_FAN_MAX keys applied to ONE digit array dig[beta][ext][n], one output per key: out[a] = sum_j sigma_a(dig_j)
// key_a,j + (sigma_a(c0) or P sigma_a(c0), 0); ginv[a] = the inverse of key a's Galois element modulo 2n.  The digits
// are read once per 8 keys.  Returns false (nothing launched) for more than 8 digits.
#define IP_FAN_MAX 64
struct IpFan {
    int n = 0;
    const u64 *key[IP_FAN_MAX] = {};
    u64 *out[IP_FAN_MAX] = {};
    unsigned ginv[IP_FAN_MAX] = {};
};
bool launch_inner_product_fanout(cm_ctx *ctx, const IpFan &f, const u64 *dig, const u64 *c0, bool c0_ext, int beta, int level,
                                 hipStream_t st);
#define IP_MULTI_KEYS 3
struct IpKeys {
    const u64 *key[IP_MULTI_KEYS] = {};
    unsigned g[IP_MULTI_KEYS] = {};
};
bool launch_inner_product_multi_key(cm_ctx *ctx, const IpBatch &b, const IpKeys &ks, int na, int beta, int level, hipStream_t st);
// out[z] = sum_j it[z].dig_j * it[0].key_j for z < nz: one key for all arrays (read once), no Galois map, no c0, no extra
// g != 0: digits and it[z].c0 (a first component in the extended basis, added as it is) through the Galois map; extra[z]
// ([2][ext][n], may be out[z]) is added
void launch_inner_product_shared_key(cm_ctx *ctx, const IpBatch &b, int beta, int level, hipStream_t st, u64 g = 0);
// out[2][ext][n] = (P c0, P c1), zero on the special limbs
void launch_raise_by_P(cm_ctx *ctx, u64 *out, const u64 *in, int level, hipStream_t st, int count = 1);   // count stacked ciphertexts
void launch_moddown_finish(cm_ctx *ctx, u64 *out, const u64 *u, const u64 *conv, const u64 *d_pinv, const u64 *addend,
                           int addend_comps, int level, u64 g, const u64 *accum, hipStream_t st, int ncomp = 2);
void launch_rescale_reduce(cm_ctx *ctx, u64 *red, const u64 *last, int ncomp, int level, hipStream_t st);
void launch_rescale_finish(cm_ctx *ctx, u64 *out, const u64 *in, const u64 *red, const u64 *d_qlinv, int ncomp, int level, hipStream_t st,
                           bool accumulate = false);
u64 rng_key(u64 seed, u64 stream);
u64 rng_draw(u64 key, u64 ctr);
void launch_sample_uniform(cm_ctx *ctx, u64 *out, const int *d_mod_idx, int limbs, u64 seed, u64 stream_base, hipStream_t st);
void launch_sample_gauss(cm_ctx *ctx, u64 *out, const int *d_mod_idx, int limbs, u64 seed, u64 stream, hipStream_t st);
void launch_evk_assemble(cm_ctx *ctx, u64 *b_out, const u64 *a_in, const u64 *e, const u64 *s_mont, const u64 *d_fac, u64 g,
                         hipStream_t st);
void launch_encrypt(cm_ctx *ctx, u64 *c0, const u64 *a, const u64 *e, const u64 *s_mont, const u64 *pt, int limbs, hipStream_t st);
void launch_decrypt(cm_ctx *ctx, u64 *out, const u64 *ct, const u64 *s_mont, int ncomp, int ct_limbs, int limbs, hipStream_t st);
// pts: all r_i*r_o plaintexts in the blocked layout written by launch_pt_block
void launch_vmm_mac(cm_ctx *ctx, u64 *out, const u64 *babies, const u64 *pts, int r_i, int r_o, int limbs, int level,
                    size_t ct_stride, int k0, int k1, hipStream_t st);
// copies plaintext (j,k) from plain[limbs][n] into the blocked array (to_blocked) or back
void launch_pt_block(cm_ctx *ctx, u64 *blocked, u64 *plain, int limbs, int r_i, int r_o, int j, int k, bool to_blocked,
                     hipStream_t st);

// Tail of a ModDown fused into the last pass of the forward transform of its converted limbs:
// for item r, component c, limb l:  out = (u - NTT(conv)) * P^{-1} (+ addend_r through the Galois map
// g_r on the first addend_comps components) (+ accum_r).  Passed to the kernel by value.
struct FinishBatch {
    int items = 0, level = 0, ext = 0, addend_comps = 0;
    int ncomp = 2, comp0 = 0;         // components handled per item, and the first of them (1, 1: second component only)
    const u64 *u[CM_KS_BATCH];        // [2][ext][n] per item (evaluation domain)
    u64 *out[CM_KS_BATCH];            // [2][level+1][n] per item
    const u64 *accum[CM_KS_BATCH];    // nullable; may alias out
    unsigned g[CM_KS_BATCH];
    const u64 *addend[CM_KS_BATCH];   // [2][level+1][n] per item, nullable; must not alias any out
    const u64 *pinv = nullptr;        // [level+1][2]: P^{-1} mod q_l and its Shoup companion
    // u_r is not stored but formed on the fly as u[r] * (mul_pt read through the Galois map mul_g[r]): the masked
    // products of a cache append, whose rescale is this tail (mul_pt[ext][n], multiplier form; nullable)
    const u64 *mul_pt = nullptr;
    unsigned mul_g[CM_KS_BATCH] = {};
};
// forward transform of conv[items*ncomp*(level+1)][n] (mods 0..level repeating) with that tail; n = 65536 only
// with src: the first pass reads row d_src_rows[i] of src for limb i (words below twice that limb's modulus) instead of conv
void launch_ntt_fwd_finish(cm_ctx *ctx, u64 *conv, const int *d_mods, const FinishBatch &fb, hipStream_t st,
                           const u64 *src = nullptr, const int *d_src_rows = nullptr);

// ops.hip internals shared with vmm.hip
bool rescale_masked_into(cm_ctx *ctx, const MulPtBatch &mb, int cnt, const u64 *pt, int level, u64 *out, hipStream_t st,
                         u64 *last, u64 *red, bool accumulate);
struct KsLevel {            // cached per level: which rows of the digit array are converted / transformed
    int level, ext, beta;
    int *d_ntt_rows = nullptr;        // rows of the [beta*ext] digit array to transform
    int *d_ntt_mods = nullptr;        // their modulus indices
    int n_ntt = 0;
    int *d_sp_rows = nullptr;         // rows level+1.. of an ext-sized array (special limbs), for both components
    int *d_sp_mods = nullptr;
    int *d_q_rows = nullptr;          // 0..level
};
const KsLevel &ks_level(cm_ctx *ctx, int level);
// digits[beta][ext][n] (evaluation domain) from evaluation-domain d[level+1][n]
// with g != 0: digits of the Galois-mapped polynomial (d is read through the permutation)
cm_status ks_raise(cm_ctx *ctx, const u64 *d, int level, u64 *digits, hipStream_t st, u64 g = 0);
// (out0, out1) = ModDown(sum_j perm_g(digits_j) * evk_j) [+ perm_g(addend) on component 0]; out = [2][level+1][n]
// addend_comps: 0 none, 1 component 0 only (rotation), 2 both (relinearisation)
cm_status ks_apply(cm_ctx *ctx, const u64 *digits, const u64 *evk, int level, u64 g, const u64 *addend,
                   int addend_comps, u64 *out, hipStream_t st, const u64 *accum = nullptr);
// out = Rot(in) (+ accum); out may alias in or accum
// extra: a [2][ext][n] sum in the extended basis that joins the key-switch sum before its ModDown
cm_status rotate_into(cm_ctx *ctx, const u64 *key, const u64 *in, int level, u64 g, u64 *out, hipStream_t st,
                      const u64 *accum = nullptr, const u64 *extra = nullptr);
// out[2][level+1][n] = ModDown(u[2][ext][n]) (+ perm_g(addend) on the first addend_comps components) (+ accum);
// the special limbs of u are overwritten
cm_status moddown_into(cm_ctx *ctx, u64 *u, int level, const u64 *addend, int addend_comps, u64 g, u64 *out,
                       const u64 *accum, hipStream_t st);
// Tables for raising component `comp` of cnt stacked ciphertexts of ncomp components at one level in
// single launches.
struct KsManyTables {
    int cnt = 0, level = 0, n_ntt = 0, ncomp = 2, comp = 1;
    int *d_src_rows = nullptr, *d_in_mods = nullptr;     // inverse transform: c1 rows of the ciphertext array, moduli
    int *d_ntt_rows = nullptr, *d_ntt_mods = nullptr;    // converted rows of the [cnt][beta][ext] digit array
};
cm_status ks_many_tables_create(cm_ctx *ctx, int level, int cnt, KsManyTables *t, int ncomp = 2, int comp = 1);
void ks_many_tables_destroy(KsManyTables *t);
// digits[k][beta][ext][n] (evaluation domain) of component t.comp of cts[k][t.ncomp][level+1][n] for k < m <= t.cnt
// (through the Galois map g if g != 0); ksin: m*(level+1) limbs of scratch
cm_status ks_raise_many(cm_ctx *ctx, const KsManyTables &t, const u64 *cts, u64 *ksin, u64 *digits, hipStream_t st,
                        int m = -1, u64 g = 0);
// outs[r][2][level+1][n] = ModDown(us + r*2*ext*n) for r < cnt (any cnt; runs in batches); special limbs of us are overwritten
// second components only: outs[r] + (level+1)*n <- ModDown(us[r][1]); the first components of us (all their limbs)
// and of outs are left as they are
cm_status moddown_many_second(cm_ctx *ctx, u64 *us, int level, int cnt, u64 *const *outs, hipStream_t st);
// out + (level+1)*n <- ModDown(R[1]) for one R = [2][ext][n], which is left untouched (its special limbs are
// transformed into a buffer of their own)
cm_status moddown_second_keep(cm_ctx *ctx, const u64 *R, int level, u64 *out, hipStream_t st);
// the same for m <= CM_KS_BATCH stacked R[r] = [2][ext][n]: outs[r] + (level+1)*n <- ModDown(R[r][1])
cm_status moddown_second_keep_many(cm_ctx *ctx, const u64 *Rs, int level, int m, u64 *const *outs, hipStream_t st);
cm_status moddown_many(cm_ctx *ctx, u64 *us, int level, int cnt, u64 *const *outs, hipStream_t st);
// one batch (m <= CM_KS_BATCH): outs[r] = ModDown(us + r*2*ext*n) + perm_g(addends[r]) on the first addend_comps
// components (+ accums[r]); addends / accums nullable arrays of nullable pointers
cm_status moddown_batch_into(cm_ctx *ctx, u64 *us, int level, int m, const u64 *const *addends, int addend_comps, u64 g,
                             const u64 *const *accums, u64 *const *outs, hipStream_t st);
// raised[r][2][ext][n] = sum_j perm_{g_r}(digits_j) * key_r + P * perm_{g_r}(in.c0): hoisted rotations left in the
// extended basis
cm_status ks_apply_many_raised(cm_ctx *ctx, const u64 *digits, int level, int cnt, const u64 *const *keys,
                               const u64 *gs, const u64 *in, u64 *const *raised, hipStream_t st, bool in_ext = false);
// out[comp][level][n] = in[comp][level+1][n] divided by q_level; up to 2*CM_KS_BATCH stacked components when the
// caller gives scratch last[ncomp][n] and red[ncomp][level][n] (up to three without)
cm_status rescale_into(cm_ctx *ctx, const u64 *in, int ncomp, int level, u64 *out, hipStream_t st, u64 *last = nullptr,
                       u64 *red = nullptr, bool accumulate = false);
u64 *arena_digits(const cm_ctx *ctx);
// room for CM_KS_BATCH key-switch sums [2][L+1+K][n] (what moddown_batch_into consumes)
u64 *arena_batch_sums(const cm_ctx *ctx);
cm_status ks_apply_many(cm_ctx *ctx, const u64 *digits, int level, int cnt, const u64 *const *keys, const u64 *gs,
                        const u64 *in, u64 *const *outs, hipStream_t st);
const u64 *find_key(const cm_evk *evk, u64 g);
// the key set was generated under the context's current CM_OPT_EVK_STORED_A setting (the kernels take the layout from it)
bool evk_fits(const cm_ctx *ctx, const cm_evk *evk);
void launch_ntt_rows(cm_ctx *ctx, u64 *data, const int *d_rows, const int *d_mods, int limbs, bool inverse, hipStream_t st);
void launch_ntt_src(cm_ctx *ctx, u64 *data, const int *d_rows, const u64 *src, const int *d_src_rows,
                    const int *d_mods, int limbs, bool inverse, hipStream_t st, u64 g = 0);
void decode_host(const cm_ctx *ctx, const std::vector<double> &m, double *re, double *im, size_t nslots);
