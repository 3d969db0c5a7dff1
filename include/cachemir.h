/*
 * libcachemir -- homomorphic vector-matrix products of one LLM decode step on one MI355X.
 *
 * The operations are those of the Cachemir paper: RNS-CKKS ciphertext operations (Sec. 2.1),
 * the packed activation-row x plaintext-matrix product with interleaved replicated packing
 * (Sec. 4.1, App. C / Algorithm 1), and the products against the encrypted KV cache with its
 * append (Sec. 5.1-5.3).  The paper treats the CKKS primitives as given; they are the
 * textbook full-RNS scheme with hybrid key switching (digits of `alpha` primes, fast
 * non-centred base conversion, floor division by the special modulus).
 *
 * Conventions
 *  - Every function returns a cm_status (0 = CM_OK, negative = error) and never throws,
 *    aborts or exits.  On error the outputs are untouched.
 *  - "host" / "device" says where a pointer must live.  A cm_ct / cm_pt is a small descriptor
 *    over CALLER-ALLOCATED device memory of cm_ct_words()/cm_pt_words() 64-bit words; the
 *    library never frees or reallocates it.  Opaque handles own their device memory and are
 *    released by the matching *_destroy.
 *  - Ring degree n (the paper's N'), S = n/2 slots (the paper's N).  Ciphertext level l has
 *    l+1 limbs.  Polynomials are stored in the evaluation (NTT) domain in an internal order;
 *    cm_ct_export() gives the canonical interchange form: coefficient domain, residues in
 *    [0, q_i), order [component][limb][coefficient].
 *  - `stream` is a hipStream_t passed as void* (0 = the null stream).  Calls that take a
 *    stream only enqueue work (kernels and device-to-device copies; no allocation, no host copy,
 *    no wait).  The others (keys, encode, encrypt, decrypt, decode, exports, plan / cache /
 *    embedding creation) run on the null stream: they first wait for all work the device has in
 *    flight and return when their result is complete.
 *  - No call reads the process environment; behaviour switches are cm_ctx_set_option() values,
 *    plan flags or cache flags, all declared here.
 *  - Randomness is a counter-based generator on 64-bit integers (SplitMix64's finaliser; stream =
 *    purpose, key id, digit, limb) so that two implementations draw identical values from a seed.
 *    It makes results reproducible; it is NOT a cryptographically secure generator.  The seed
 *    passed to cm_keygen_rotations / cm_encrypt is public (the uniform halves are its streams and
 *    can be recomputed from the key or ciphertext); the error polynomials are drawn from the
 *    streams of that seed XOR a 64-bit value derived from the SECRET key's seed, which must
 *    therefore be kept private and must not be reused as a public seed.
 *  - A context's scratch arena is shared by all calls on it: calls on one context must not
 *    overlap in time (enqueue them on one stream, or order the streams).  A plan, a cache and
 *    a rotary-embedding object each hold one work area of their own with the same rule.
 *  - The hot calls (cm_rotate*, cm_vmm_pt*, cm_vmm_kv, cm_kv_append, cm_rope_apply and the
 *    element-wise ones) allocate nothing and only enqueue kernels and device copies once the
 *    per-level tables exist (the first call at a level builds them), so they can be captured
 *    into a HIP graph after one eager call.
 */
#ifndef CACHEMIR_H
#define CACHEMIR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cm_status;
enum {
    CM_OK = 0,
    CM_E_INVAL = -1,   /* bad argument (null pointer, size, unsupported ring degree) */
    CM_E_LEVEL = -2,   /* no level left, or operand levels differ */
    CM_E_SCALE = -3,   /* operand scales differ */
    CM_E_NOKEY = -4,   /* rotation step or relinearisation key not generated */
    CM_E_LAYOUT = -5,  /* plan / cache / ciphertext shapes do not fit together */
    CM_E_NOMEM = -6,   /* device or host allocation failed */
    CM_E_HIP = -7,     /* a HIP call failed; see cm_last_hip_error() */
    CM_E_TOOBIG = -8   /* the operand exceeds the fixed work area of an entry point that allocates nothing */
};
const char *cm_strerror(cm_status s);
int32_t cm_last_hip_error(void);

/* Parameter set.  The modulus chain is derived inside the library by the rule
 *   candidates 2^bits + 1 - k*2n (k = 1,2,..), primes kept in order:
 * q_0 from q0_bits, q_1..q_{n_q-1} from qi_bits (one scan: if q0_bits == qi_bits the chain is
 * the first n_q primes of that scan), special primes p_0..p_{n_p-1} from p_bits.
 * alpha = primes per key-switch digit (alpha <= 8 and n_p <= 8, n_q + n_p <= 64, at most 16 digits;
 * anything else is CM_E_INVAL).  hamming = 0: i.i.d. uniform ternary secret, else the
 * exact number of non-zero secret coefficients.  sigma must be 3.2 (error table is fixed). */
typedef struct {
    int32_t n;          /* ring degree: 4096 or 65536 */
    int32_t n_q;        /* ciphertext primes (top level L = n_q - 1) */
    int32_t n_p;        /* special primes K */
    int32_t alpha;      /* primes per digit */
    int32_t q0_bits, qi_bits, p_bits;
    int32_t hamming;
    double scale;       /* default encoding scale Delta */
    double sigma;
} cm_params;

typedef struct cm_ctx cm_ctx;
typedef struct cm_sk cm_sk;
typedef struct cm_evk cm_evk;
typedef struct cm_vmm_plan cm_vmm_plan;
typedef struct cm_kv cm_kv;

typedef struct {
    uint64_t *dev;      /* device: ncomp * (level+1) * n words */
    int32_t level;
    int32_t ncomp;      /* 2, or 3 before relinearisation */
    double scale;
} cm_ct;

typedef struct {
    uint64_t *dev;      /* device: (level+1) * n words */
    int32_t level;
    int32_t mont;       /* 1: stored pre-multiplied by 2^64 mod q_i (multiplier operand form) */
    double scale;
} cm_pt;

/* ---- context ------------------------------------------------------------------------ */
/* Builds primes, roots, twiddle and conversion tables and uploads them; allocates the scratch
 * arena.  Uses the current HIP device. */
cm_status cm_ctx_create(const cm_params *p, cm_ctx **out);
void cm_ctx_destroy(cm_ctx *ctx);
/* Behaviour switches of a context (host call, takes effect for later calls; unknown option: CM_E_INVAL).
 *   CM_OPT_EVK_STORED_A  value != 0: evaluation keys generated from now on keep BOTH halves in device
 *     memory (b_j and a_j, 2 (L+1+K) n words per digit) and the key-switch kernels read a_j; 0 (default):
 *     only b_j is kept and the kernels regenerate a_j from its stream.  Same residues either way, hence
 *     bit-identical results.  A key set can only be used while the option has the value it was generated
 *     under (else CM_E_INVAL).
 *   CM_OPT_TWO_STEP_MASKS  value != 0: cm_kv_append(_group) forms its masked products as stored
 *     ciphertexts and rescales them afterwards, instead of forming them inside the rescale's transform
 *     (n = 65536 only; a cross-check of that fused path, bit-identical results). */
enum { CM_OPT_EVK_STORED_A = 1, CM_OPT_TWO_STEP_MASKS = 2 };
cm_status cm_ctx_set_option(cm_ctx *ctx, int32_t option, int32_t value);
/* host out[n_q + n_p]: q_0..q_L then p_0..p_{K-1}. */
cm_status cm_ctx_moduli(const cm_ctx *ctx, uint64_t *out);
size_t cm_ct_words(const cm_ctx *ctx, int32_t level, int32_t ncomp);
size_t cm_pt_words(const cm_ctx *ctx, int32_t level);
/* host out[19]: the cumulative table of the error sampler (for cross-checks). */
cm_status cm_ctx_gauss_table(const cm_ctx *ctx, uint64_t *out);

/* ---- keys (Sec. 2.1 rotation / ct-ct multiplication need them; client side) ---------- */
cm_status cm_keygen_secret(cm_ctx *ctx, uint64_t seed, cm_sk **out);
void cm_sk_destroy(cm_sk *sk);
/* host out[n]: secret coefficients in {-1,0,1}. */
cm_status cm_sk_coeffs(const cm_ctx *ctx, const cm_sk *sk, int8_t *out);
/* Keys for left rotations by steps[i] slots (negative = right), and for s^2 -> s if
 * with_relin.  Steps with equal Galois element share a key.  A key is (b_j, a_j) per digit with
 * b_j = -a_j s + e_j + P s_from on the digit's own limbs; a_j is uniform and drawn directly in the
 * evaluation domain (its value at psi^(2k+1) is draw brev(k) of the counter-based generator's stream
 * for (seed, key, digit, limb)), so only the b_j are kept in device memory, (L+1+K) n words per
 * digit, and the kernels regenerate a_j where they use it (CM_OPT_EVK_STORED_A keeps a_j too).  `seed`
 * is public; e_j is drawn from the streams of seed XOR the secret key's private value. */
cm_status cm_keygen_rotations(cm_ctx *ctx, const cm_sk *sk, const int32_t *steps, size_t nsteps,
                              int32_t with_relin, uint64_t seed, cm_evk **out);
void cm_evk_destroy(cm_evk *evk);
/* Canonical (coefficient-domain, plain residues) copy of one key polynomial to host
 * out[(L+1+K)*n]: step = rotation step (ignored if relin != 0), comp 0 = b, 1 = a (regenerated). */
cm_status cm_evk_export(cm_ctx *ctx, const cm_evk *evk, int32_t step, int32_t relin,
                        int32_t digit, int32_t comp, uint64_t *out);

/* ---- encode / encrypt / decrypt (client side, Sec. 2.1 last paragraph) ---------------- */
/* Integer coefficients round(scale * m_k) of the polynomial whose slot values are
 * re[j] + i*im[j] (im may be NULL; slots past nslots are 0).  host in, host out[n]. */
cm_status cm_encode_coeffs(const cm_ctx *ctx, const double *re, const double *im, size_t nslots,
                           double scale, int64_t *out);
/* Signed coefficients (host, n of them) -> plaintext in out->dev.  out->dev, out->mont must be
 * set by the caller; level and scale are written. */
cm_status cm_pt_from_coeffs(cm_ctx *ctx, const int64_t *coeffs, int32_t level, double scale,
                            cm_pt *out);
cm_status cm_encode(cm_ctx *ctx, const double *re, const double *im, size_t nslots,
                    int32_t level, double scale, cm_pt *out);
/* Symmetric encryption (c0, c1) = (-a s + e + m, a); pt must have mont == 0.  a: streams of `seed` (public),
 * e: streams of seed XOR the secret key's private value. */
cm_status cm_encrypt(cm_ctx *ctx, const cm_sk *sk, const cm_pt *pt, uint64_t seed, cm_ct *out);
/* c0 + c1 s (+ c2 s^2) on the lowest min(level,1)+1 limbs -> out (mont = 0). */
cm_status cm_decrypt(cm_ctx *ctx, const cm_sk *sk, const cm_ct *ct, cm_pt *out);
/* Slot values of a plaintext of level <= 1.  host re/im[nslots] (im may be NULL). */
cm_status cm_decode(cm_ctx *ctx, const cm_pt *pt, double *re, double *im, size_t nslots);
/* Canonical form to host out[ncomp*(level+1)*n]. */
cm_status cm_ct_export(cm_ctx *ctx, const cm_ct *ct, uint64_t *out);
cm_status cm_pt_export(cm_ctx *ctx, const cm_pt *pt, uint64_t *out);

/* ---- ciphertext operations of Sec. 2.1 ------------------------------------------------ */
cm_status cm_add(cm_ctx *ctx, const cm_ct *a, const cm_ct *b, cm_ct *out, void *stream);
/* out = a * pt (pt->mont must be 1); scale multiplies, level unchanged (rescale separately).  Level 0
 * (nothing left to rescale into): CM_E_LEVEL, as for cm_mul_ct. */
cm_status cm_mul_pt(cm_ctx *ctx, const cm_ct *a, const cm_pt *pt, cm_ct *out, void *stream);
/* Tensor product, three components, not relinearised. */
cm_status cm_mul_ct(cm_ctx *ctx, const cm_ct *a, const cm_ct *b, cm_ct *out, void *stream);
cm_status cm_relinearize(cm_ctx *ctx, const cm_evk *evk, const cm_ct *a, cm_ct *out, void *stream);
/* Division by the last prime (floor variant): level drops by one. */
cm_status cm_rescale(cm_ctx *ctx, const cm_ct *a, cm_ct *out, void *stream);
/* cm_rescale for callers that cannot allocate device memory at all (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): the same result, bit for bit, but nothing is taken from
 * the context's arena or from per-level tables (which an ordinary call builds, and allocates, the first time a
 * level is used).  Its work area is a fixed 32 MiB device array inside the library (one per GPU, held until
 * the process ends), so ncomp * (level + 1) * n may be at most 4 Mi words (n = 65536: two components up to
 * level 31, three up to level 20): beyond that CM_E_TOOBIG and nothing is enqueued.  out must not alias a.
 * The call only enqueues kernels on `stream`; it calls no allocator.  All calls on one GPU share the work area:
 * calls that may overlap in time (different streams without ordering, different contexts) race. */
cm_status cm_rescale_static(cm_ctx *ctx, const cm_ct *a, cm_ct *out, void *stream);
cm_status cm_level_drop(cm_ctx *ctx, const cm_ct *a, int32_t level, cm_ct *out, void *stream);
/* Rot(in, step)[i] = in[i + step]: Galois map, then key switch of the second component. */
cm_status cm_rotate(cm_ctx *ctx, const cm_evk *evk, const cm_ct *in, int32_t step, cm_ct *out,
                    void *stream);
/* nsteps rotations of ONE ciphertext that share the raised digits of its second component
 * (the map is applied after raising, so limbs differ from cm_rotate's; both are valid). */
cm_status cm_rotate_hoisted(cm_ctx *ctx, const cm_evk *evk, const cm_ct *in, const int32_t *steps,
                            size_t nsteps, cm_ct *outs, void *stream);

/* ---- packed plaintext product (Sec. 4.1, Algorithm 1) ---------------------------------- */
/* W: host, row-major d_in x d_out.  One of d_in == d_out, d_out = alpha*d_in, d_in =
 * alpha*d_out (alpha a power of two); S/min(d) and S/max(d) must be integers.  r_i = baby
 * steps (0 = default: the power of two at or just above sqrt of the diagonal count, twice that
 * for the forms that keep the baby steps in the extended basis and for token-batched plans, whose
 * baby steps are several times cheaper than their giant steps); tau = residue the outputs land on
 * (0, or the slot residue of a token about to be appended to the cache).  The weight diagonals
 * are encoded at `pt_scale` (0 = the context scale) for input level `level` and stay on the
 * device.  Layouts: input element a at slot a*t (d_in <= d_out) or (a%d)*t + (a/d)*t'
 * (d_in > d_out); output element c at slot c*t + tau, or (c%d)*t + (c/d)*t' + tau when
 * expanding; d = min(d_in, d_out), t = S/d, t' = S/max(d_in, d_out). */
cm_status cm_vmm_plan_create(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i, int32_t tau,
                             int32_t level, double pt_scale, const double *W, cm_vmm_plan **out);
/* Same, from already rounded integer coefficients of the r_i*r_o diagonals:
 * coeffs[(j*r_o + k)*n + c], host. */
cm_status cm_vmm_plan_create_from_coeffs(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i,
                                         int32_t tau, int32_t level, double pt_scale,
                                         const int64_t *coeffs, cm_vmm_plan **out);
/* General form: exactly one of W (as in cm_vmm_plan_create) and coeffs (as in
 * cm_vmm_plan_create_from_coeffs) is non-null.  flags:
 *   CM_VMM_RAISED_SUMS  the hoisted baby-step rotations (App. C: the r_i - 1 rotations of one
 *     ciphertext) are not divided by the special modulus P one by one: they stay on the
 *     level+1+K limbs of the extended basis as (u0 + P sigma(c0), u1), the plaintext products are
 *     summed there, and each sum is divided by P inside the giant step that consumes it.  Same
 *     rotations, same plaintext products, r_i - 1 fewer ModDowns; the weight plaintexts take
 *     level+1+K limbs each.  The result differs from the plain form by rounding noise only.
 *   CM_VMM_DIRECT_GIANTS  (implies CM_VMM_RAISED_SUMS) the giant steps of Algorithm 1 are unrolled:
 *     y' = inner_0 + sum_{k>=1} Rot(inner_k, k G) instead of the nested Rot(.. + Rot(inner_{r_o-1}, G), G).
 *     Same number of rotations, but they are independent: their ModUps run as one batch, and all of
 *     them share one ModDown.  Only the second component of inner_k is divided by P (for the digits);
 *     the first joins the sum through the Galois map on all limbs of the extended basis.  Needs the r_o - 1 keys of k G (cm_vmm_plan_steps lists them)
 *     instead of the single key of G.
 *   CM_VMM_TOKEN_BATCH  the prompt phase (Sec. 5.4): the ciphertext holds t = S/d tokens, element b
 *     of token tau at slot b*t + tau, and y holds the t rows of X W in the same layout.  No
 *     preprocess and no reduce rotations; all d diagonals (each repeated over the residues), baby
 *     step j*t, giant step r_i*t, r_i*r_o = d; d_in == d_out (a wider or taller matrix is a set of
 *     square ones, cm_vmm_pt_multi shares their baby steps), tau = 0.  Combines with the other two.
 *   CM_VMM_UNROLLED_LADDERS  (implies CM_VMM_DIRECT_GIANTS) the two rotate-and-add ladders of
 *     Algorithm 1 (preprocess: c <- c + Rot(c, 2^i (t-1)); reduce: c <- c + Rot(c, +-2^l)) are unrolled
 *     in ceil(L/3) runs of as equal length as possible: a run of g steps equals c + the rotations of
 *     c by the 2^g - 1 non-empty subset sums of its steps, which are rotations of ONE ciphertext and
 *     share its raised digits.  The whole
 *     product then stays in the extended basis: one ModDown of both components at its end, second
 *     components alone divided by P where digits are needed.  More rotations and keys (7 per run of
 *     three steps instead of 3; cm_vmm_plan_steps lists them), fewer ModUps and ModDowns.
 * Unknown flag bits: CM_E_INVAL. */
enum { CM_VMM_RAISED_SUMS = 1, CM_VMM_DIRECT_GIANTS = 2, CM_VMM_TOKEN_BATCH = 4, CM_VMM_UNROLLED_LADDERS = 8 };
cm_status cm_vmm_plan_create_ex(cm_ctx *ctx, int32_t d_in, int32_t d_out, int32_t r_i, int32_t tau,
                                int32_t level, double pt_scale, const double *W,
                                const int64_t *coeffs, uint32_t flags, cm_vmm_plan **out);
void cm_vmm_plan_destroy(cm_vmm_plan *plan);
/* Rotation steps the plan uses: returns their number, writes up to cap of them (host). */
int32_t cm_vmm_plan_steps(const cm_vmm_plan *plan, int32_t *steps, int32_t cap);
/* r_i, r_o, rotation count.  The integer coefficients are not kept; cm_vmm_plan_diag_export
 * writes the encoded diagonal (j, k) in canonical plain residues to host out[limbs*n], limbs =
 * level+1 (plus the K special limbs for a CM_VMM_RAISED_SUMS plan). */
cm_status cm_vmm_plan_info(const cm_vmm_plan *plan, int32_t *r_i, int32_t *r_o, int32_t *n_rot);
cm_status cm_vmm_plan_diag_export(cm_ctx *ctx, const cm_vmm_plan *plan, int32_t j, int32_t k,
                                  uint64_t *out);
/* y = x W.  x at the plan's level; y one level lower, scale x.scale*pt_scale/q_level.  Slots
 * other than the output slots hold partial sums (masking is left to the next layer, Sec. 4.2). */
cm_status cm_vmm_pt(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *plan, const cm_ct *x,
                    cm_ct *y, void *stream);

/* Several products of the same input (the q / k / v projections of a token, or gate and up):
 * ys[i] = x W_i for plans of one shape (same d_in, d_out, level, r_i; the output residue tau may
 * differ), all created with CM_VMM_RAISED_SUMS.  The preprocess rotations and the hoisted baby
 * steps depend on x only, so they run once; each plan then does its own products and giant
 * steps.  Every ys[i] is bit for bit what cm_vmm_pt(plans[i], x) gives.  plans must be distinct. */
cm_status cm_vmm_pt_multi(cm_ctx *ctx, const cm_evk *evk, const cm_vmm_plan *const *plans,
                          int32_t nplans, const cm_ct *x, cm_ct *const *ys, void *stream);

/* ---- encrypted KV cache (Sec. 5) -------------------------------------------------------- */
/* CM_QK_GROUP: query-times-K for a query GROUP (Sec. 5.4: token tau at residue tau of every (e, h)
 * block, possibly after an inner rotation): nothing is replicated, and slot (c, h, tau') of the
 * result is the score of the query at residue tau' against key token c*t + tau'.
 * CM_SV_GROUP: scores-times-V for such scores: the residues are NOT summed; slot (e, h, tau') of the
 * result is sum_c s[c, h, tau'] V[c*t + tau', h, e], the contribution of the keys at residue tau' to
 * the query whose scores sit there.  An inner rotation by t - delta takes it back to the query's own
 * residue; the sum over delta is the attention output of the whole group. */
enum { CM_QK = 0, CM_SV = 1, CM_QK_GROUP = 2, CM_SV_GROUP = 3,
       CM_KV_INDEX = 4 /* cm_kv_load / cm_kv_export only: a ciphertext of the key index */ };
/* Cache for `heads` heads of `dim` dims (heads*dim*t = S) holding up to max_tokens tokens
 * (<= dim*t) at ciphertext level `level` and scale `scale`.  r_i = baby steps of the
 * score-times-V product (0 = dim, no giant steps).  A head count that is not a power of two (GPT2-base:
 * 12) is padded to the next one, Hp: the layout is slot (e, h, tau) = (e*Hp + h)*t + tau with t = S/(Hp*dim),
 * the padding heads hold zeros (the same holds for cm_rope_create). */
cm_status cm_kv_create(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t r_i, int32_t level,
                       double scale, int32_t max_tokens, cm_kv **out);
/* flags: CM_KV_UNROLLED_LADDERS — in query-times-K the sum over the dims of every head (Sec. 5.1 step 2,
 * a rotate-and-add ladder of log2(dim) dependent rotations per key ciphertext) is computed in the
 * extended basis: the ladder is cut into ceil(L/3) runs, a run of g steps adds the 2^g - 1 hoisted
 * rotations by its subset sums (one ModUp per run), one ModDown ends it.  scores-times-V takes the
 * same form: its giant steps are unrolled (sum_g Rot(inner_g, g G), one key per multiple of the giant
 * step) and its ladder over the residues runs in the extended basis before the one ModDown and the
 * rescale.  More rotation keys (cm_kv_steps lists them), fewer ModUps and ModDowns.  Unknown bits:
 * CM_E_INVAL. */
/* CM_KV_KEY_INDEX — next to the K cache of Sec. 5.1 the cache keeps a re-layout of it, the key index: `dim`
 * ciphertexts X_{g r_i + j} = sum_c Rot(mask_c, -g r_i B) Rot(K_c, j B) (B = heads * t slots per copy), i.e. copy b of
 * X_{g r_i + j} holds dim (b + j) mod dim of key group (b - g r_i) mod dim.  Sec. 5.1's scores
 *   sum_c mask_c sum_k Rot(q . K_c, k B)  =  sum_k Rot(q, k B) . D_k,   D_k = sum_c mask_c Rot(K_c, k B)
 * (Rot(a b) = Rot(a) Rot(b)), a diagonal product like scores-times-V (Sec. 5.2) whose baby-step / giant-step
 * schedule runs on the index as it is: r_i - 1 hoisted rotations of the query, dim products, dim / r_i
 * relinearisations and giant steps for the WHOLE cache, no mask afterwards: query-times-K then returns the
 * scores ONE level below the cache (not two) and costs what scores-times-V costs.  The price is paid at
 * append: r_i - 1 more hoisted rotations (of the new key) and `dim` more masked products per token or token
 * group, and `dim` more ciphertexts of memory.  cm_kv_load(CM_QK) does not update the index (that would
 * cost a level): load its ciphertexts with CM_KV_INDEX.  With the index, cm_kv_steps lists no rotation for
 * the sum over the dims and cm_kv_set_shared_dims has no effect on query-times-K. */
enum { CM_KV_UNROLLED_LADDERS = 1, CM_KV_KEY_INDEX = 2 };
cm_status cm_kv_create_ex(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t r_i, int32_t level,
                          double scale, int32_t max_tokens, uint32_t flags, cm_kv **out);
/* Sec. 5.1 sums the product of every key ciphertext over all dim copies and then keeps copy e = c by a mask.
 * Because Rot(a b) = Rot(a) Rot(b), the mask can be applied before the last `shared` terms of that sum
 * (dim = shared * E2, B = heads * t slots per copy):
 *   sum_c mask_c sum_{k < dim} Rot(P_c, k B) = sum_{k1 < shared} Rot( sum_c mask_{c+k1} T_c, k1 B ),
 *   T_c = sum_{k2 < E2} Rot(P_c, k2 shared B),
 * which takes shared - 1 rotations for the WHOLE cache (plus nk * shared plaintext products by the dim
 * slot rotations of the mask) instead of log2(shared) ladder steps per key ciphertext.  Same scores,
 * same levels.  shared = 1 (the default) is the printed order; shared = dim removes every
 * per-ciphertext rotation and pays off for long contexts.  Only for caches created with
 * CM_KV_UNROLLED_LADDERS (else CM_E_INVAL); shared a power of two <= dim (else CM_E_LAYOUT).
 * Allocates max_tokens / t + shared + dim ciphertext-sized buffers (CM_E_NOMEM leaves shared = 1)
 * and changes the rotation amounts cm_kv_steps lists.  Not to be called while a product of this cache
 * is in flight. */
cm_status cm_kv_set_shared_dims(cm_kv *kv, int32_t shared);
void cm_kv_destroy(cm_kv *kv);
int32_t cm_kv_steps(const cm_kv *kv, int32_t *steps, int32_t cap);
int32_t cm_kv_tokens(const cm_kv *kv);
/* Install an already packed cache ciphertext (which = CM_QK: K ciphertext idx; CM_SV: V
 * ciphertext idx) and set the token count. */
cm_status cm_kv_load(cm_ctx *ctx, cm_kv *kv, int32_t which, int32_t idx, const cm_ct *ct,
                     void *stream);
cm_status cm_kv_set_tokens(cm_kv *kv, int32_t ntok);
cm_status cm_kv_export(cm_ctx *ctx, const cm_kv *kv, int32_t which, int32_t idx, uint64_t *out);
/* Every mask the cache uses is a slot rotation of one of three base masks, applied as the
 * Galois permutation of the encoded base.  This replaces a base by given integer coefficients
 * (host, n of them; encoding scale = the prime the following rescale removes): kind 0 = slots
 * (0, h, tau) for all h, tau, at level-1 (keeps one copy of the replicated scores, Sec. 5.1 step
 * 3); kind 1 = slots of residue 0 at level+1 (K append); kind 2 = slots (0, h, 0) at level+1 (V
 * append, Sec. 5.2); kind 3 = every slot and kind 4 = slots (0, h, tau) for all h, tau, both at
 * level+1 (cm_kv_append_group).  For callers that need bit-identical plaintexts on two
 * implementations. */
cm_status cm_kv_set_mask(cm_kv *kv, int32_t kind, const int64_t *coeffs);
/* Append the next token: k_new / v_new hold the new vectors at residue tau = ntok mod t, one
 * level above the cache; they are masked (one plaintext product each) and added. */
cm_status cm_kv_append(cm_ctx *ctx, const cm_evk *evk, cm_kv *kv, const cm_ct *k_new,
                       const cm_ct *v_new, void *stream);
/* Cache generation in the prompt phase (Sec. 5.4): append the next t tokens at once.  k_grp /
 * v_grp hold token ntok + tau at residue tau of every (e, h) block (what a CM_VMM_TOKEN_BATCH
 * product with (e, h)-ordered columns, then the rotary embedding with tau = -1, leaves), one level
 * above the cache; ntok must be a multiple of t (else CM_E_LAYOUT).  k_grp becomes K ciphertext
 * ntok/t (one product with the all-ones mask keeps level and scale equal to the one-token
 * append); every V ciphertext takes one block row of v_grp by one masked product, all residues
 * together.  Same rotation keys as cm_kv_append. */
cm_status cm_kv_append_group(cm_ctx *ctx, const cm_evk *evk, cm_kv *kv, const cm_ct *k_grp,
                             const cm_ct *v_grp, void *stream);
/* which = CM_QK: in = query at (e, h, 0) slots, cache level; out = scores, two levels lower (one level lower
 * for a cache with CM_KV_KEY_INDEX).
 * which = CM_SV: in = scores; out = attention output at (e, h, 0), one level lower.
 * CM_QK_GROUP / CM_SV_GROUP: the same levels; no keys for the residue rotations are needed. */
cm_status cm_vmm_kv(cm_ctx *ctx, const cm_evk *evk, const cm_kv *kv, int32_t which,
                    const cm_ct *in, cm_ct *out, void *stream);

/* ---- grouped-query attention on a cache that stores every KV head once -------------------------------
 * The paper packs one K / V head per query head (Sec. 5.3).  For a model whose `heads` KV heads are each shared by
 * `group` query heads, create the cache with cm_kv_create(heads = KV heads): it then holds t_kv = S/(heads*dim)
 * tokens per K ciphertext and dim*t_kv tokens in all (4096 for 8 x 128 on 2^15 slots), 1/group of the memory and of
 * the append work of a cache with every KV head repeated.  The query and the attention output use the layout of
 * H = group*heads heads (t = t_kv/group), head h = hk*group + g, whose slot (e, h, tau) IS slot (e, hk, g*t + tau)
 * of the cache layout.  A query head meets all t_kv token residues of its KV head in `group` passes: in pass delta
 * the replicated query is moved by the inner rotation (Sec. 5.4) of delta*t residues and multiplied into the cache
 * as a query group (CM_QK_GROUP).  scores[delta] (an array of `group` ciphertexts, two levels below the cache; one
 * level below it for a cache with CM_KV_KEY_INDEX, whose passes run on the index at the cost of scores-times-V)
 * holds at slot (c, hk, j) the score of head (hk, (j/t - delta) mod group) against token c*t_kv + j.
 * cm_gqa_sv takes `group` score ciphertexts in that layout at the cache level, runs scores-times-V per pass
 * without the sum over the residues (CM_SV_GROUP), moves each result back by (group - delta)*t residues, adds them
 * and sums the t residues of a run: Att[h, e] at (e, h, 0), two levels below the cache.
 * cm_gqa_create: kv must outlive the object; group a power of two dividing t_kv (else CM_E_LAYOUT); coeffs
 * (nullable, host [2][group-1][3][n]): integer coefficients of the plaintexts of the inner rotations by delta*t,
 * delta = 1..group-1, first those applied to the query (level+1), then those applied to the results (level-1), each
 * as cm_inner_rot_create takes them.  cm_gqa_steps lists the rotations needed beyond those of cm_kv_steps that are
 * multiples of t_kv (no other step of the cache is used).  q: (e, h, 0) layout, one level above the cache. */
typedef struct cm_gqa cm_gqa;
cm_status cm_gqa_create(cm_ctx *ctx, const cm_kv *kv, int32_t group, const int64_t *coeffs, cm_gqa **out);
void cm_gqa_destroy(cm_gqa *gqa);
int32_t cm_gqa_steps(const cm_gqa *gqa, int32_t *steps, int32_t cap);
cm_status cm_gqa_qk(cm_ctx *ctx, const cm_evk *evk, const cm_gqa *gqa, const cm_kv *kv, const cm_ct *q, cm_ct *scores,
                    void *stream);
cm_status cm_gqa_sv(cm_ctx *ctx, const cm_evk *evk, const cm_gqa *gqa, const cm_kv *kv, const cm_ct *scores, cm_ct *out,
                    void *stream);

/* ---- rotary embedding with the extraction fused (Sec. 4.2, App. D) ------------------------ */
/* The element-wise layer after the q / k projections: for token `token`, every pair of dims
 * (2m, 2m+1) of every head is turned by token * base^(-2m/dim), and every slot that is not a
 * valid slot (e, h, tau) = (e*heads + h)*t + tau comes out zero, whatever partial sums the
 * projection left there.  Three plaintext products, two rotations (by +-heads*t slots), one
 * level; the plaintexts are encoded at the scale of the prime the rescale removes, so y keeps
 * the scale of x.  coeffs (nullable, host [3][n]): integer coefficients of p0, p1, p2 to use
 * instead of the library's own encoding, for callers that need bit-identical plaintexts on two
 * implementations.  x at `level`, y one level lower; y must not alias x.
 * tau = -1: x holds t tokens, token `token` + r at residue r (the prompt phase, Sec. 5.4), and
 * every residue is turned by the angles of its own token. */
typedef struct cm_rope cm_rope;
cm_status cm_rope_create(cm_ctx *ctx, int32_t heads, int32_t dim, int32_t level, int32_t token,
                         int32_t tau, double base, const int64_t *coeffs, cm_rope **out);
void cm_rope_destroy(cm_rope *rope);
/* Rotation steps it needs: returns 2, writes up to cap of them (host). */
int32_t cm_rope_steps(const cm_rope *rope, int32_t *steps, int32_t cap);
cm_status cm_rope_apply(cm_ctx *ctx, const cm_evk *evk, const cm_rope *rope, const cm_ct *x,
                        cm_ct *y, void *stream);
/* Inner rotation (Sec. 5.4, the prompt-phase Q K^T): y[b*t + tau'] = x[b*t + (tau' - delta) mod t]
 * for every block b of t consecutive slots, 0 < delta < t, t a power of two.  Two masked products
 * (mask before rotation, encoded at the scale of the prime the rescale removes), rotations by
 * -delta and t - delta, one level: the same object and calls as the embedding (cm_rope_steps,
 * cm_rope_apply, cm_rope_destroy).  coeffs (nullable, host [3][n]): integer coefficients of the zero
 * plaintext, the mask of the residues >= t - delta and the mask of the residues < t - delta. */
cm_status cm_inner_rot_create(cm_ctx *ctx, int32_t t, int32_t delta, int32_t level,
                              const int64_t *coeffs, cm_rope **out);

/* ---- building blocks exposed for measurement and parity -------------------------------- */
/* Forward / inverse negacyclic NTT of `limbs` limbs in place (device), limb i under modulus
 * index mod_idx[i] (host array, read before the call returns; indices into q_0..q_L,p_0..);
 * 1 <= limbs <= 1024.  Enqueues only (a list that is not a run of consecutive indices is written into
 * a per-context staging array by a small kernel: two such calls on different streams must be ordered). */
cm_status cm_ntt(cm_ctx *ctx, uint64_t *dev, const int32_t *mod_idx, int32_t limbs,
                 int32_t inverse, void *stream);
/* One hybrid key switch of an evaluation-domain polynomial d[level+1][n] (device) with the key
 * of rotation `step` (or the relinearisation key): ks0, ks1 device [level+1][n]. */
cm_status cm_keyswitch(cm_ctx *ctx, const cm_evk *evk, int32_t step, int32_t relin,
                       const uint64_t *d, int32_t level, uint64_t *ks0, uint64_t *ks1,
                       void *stream);

/* Per-kernel-family timing: while enabled, every launch of the listed families is bracketed by
 * HIP events on its own stream.  cm_profile_enable(ctx, 1) clears the records and starts,
 * (ctx, 0) stops; cm_profile_get sums launches, work units (limbs for the NTTs, written limbs for
 * base conversion and element-wise kernels, 1 otherwise) and milliseconds of one family. */
enum {
    CM_K_NTT_FWD = 0, CM_K_NTT_INV = 1, CM_K_BASE_CONV = 2, CM_K_INNER_PRODUCT = 3,
    CM_K_MODDOWN_FINISH = 4, CM_K_VMM_MAC = 5, CM_K_ELEMENTWISE = 6, CM_K_RESCALE = 7,
    CM_K_FAMILIES = 8
};
cm_status cm_profile_enable(cm_ctx *ctx, int32_t on);
cm_status cm_profile_get(cm_ctx *ctx, int32_t family, double *launches, double *units, double *ms);

/* Streaming-bandwidth probe (a measurement aid, not part of the method; for callers that report a kernel's rate
 * against what the device's memory system gives a plain kernel of the same read/write mix): runs a plain streaming
 * kernel `reps` times over about `bytes` bytes of its own device buffers (64 MiB .. 16 GiB, allocated and freed
 * inside; null stream, synchronous) and returns the best rate in GB/s (10^9 bytes) of bytes read plus bytes written.
 *   CM_PROBE_READ          one contiguous run per workgroup, 16-byte non-temporal loads (the plaintext stream of the
 *                          packed product, the key stream of an inner product)
 *   CM_PROBE_COPY          one read stream, one write stream (the two passes of a transform)
 *   CM_PROBE_READ3_WRITE1  three read streams, one write stream (an inner product that writes its rotated outputs)
 * Errors: CM_E_INVAL (arguments), CM_E_NOMEM, CM_E_HIP. */
enum { CM_PROBE_READ = 0, CM_PROBE_COPY = 1, CM_PROBE_READ3_WRITE1 = 2 };
cm_status cm_hbm_probe(int32_t kind, uint64_t bytes, int32_t reps, double *gb_per_s);

#ifdef __cplusplus
}
#endif
#endif
