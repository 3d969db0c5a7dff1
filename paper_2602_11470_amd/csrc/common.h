// Internal declarations of libcachemir: modular limb arithmetic for gfx950, context tables
// and kernel launchers.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <new>
#include <vector>

#include "../../include/cachemir.h"

typedef uint64_t u64;
typedef unsigned __int128 u128;

// ---- 64-bit modular arithmetic -----------------------------------------------------------
// All moduli are below 2^62.  Three multiplier forms are used:
//   Shoup:      constant w with companion wp = floor(w 2^64 / q); result in [0, 2q) (lazy).
//   Montgomery: one operand pre-multiplied by 2^64 mod q; products are accumulated in 128
//               bits and reduced once (REDC), result in [0, q).
struct ModC {
    u64 q;
    u64 qinv;   // q^{-1} mod 2^64
    u64 r2;     // 2^128 mod q
};

__host__ __device__ __forceinline__ u64 mulhi64(u64 a, u64 b) {
#ifdef __HIP_DEVICE_COMPILE__
    return __umul64hi(a, b);
#else
    return (u64)(((u128)a * b) >> 64);
#endif
}

// a*w mod q in [0, 2q) for any a < 2^64
__device__ __forceinline__ u64 mul_shoup_lazy(u64 a, u64 w, u64 wp, u64 q) {
    return a * w - mulhi64(a, wp) * q;
}
__device__ __forceinline__ u64 mul_shoup(u64 a, u64 w, u64 wp, u64 q) {
    u64 r = mul_shoup_lazy(a, w, wp, q);
    return r >= q ? r - q : r;
}
// T 2^-64 mod q in [0, q), for T with (T >> 64) < q
__device__ __forceinline__ u64 redc(u128 T, u64 q, u64 qinv) {
    u64 lo = (u64)T, hi = (u64)(T >> 64);
    u64 t = mulhi64(lo * qinv, q);
    u64 r = hi - t;
    return hi < t ? r + q : r;
}
// a 2^64 mod q
__device__ __forceinline__ u64 to_mont(u64 a, const ModC &m) { return redc((u128)a * m.r2, m.q, m.qinv); }
__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 q) {
    u64 s = a + b;
    return s >= q ? s - q : s;
}
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

// Position i of the evaluation order holds the value at psi^(2 brev(i) + 1); the Galois map
// X -> X^g moves the value at exponent e*g to exponent e: out[i] = in[perm_src(i, g)].  It maps
// aligned blocks of 2^k positions onto aligned blocks (and i^1 to src^1).
__device__ __forceinline__ unsigned perm_src(unsigned i, unsigned g, int logn) {
    unsigned e = 2u * (__brev(i) >> (32 - logn)) + 1u;
    unsigned s = (e * g) & ((2u << logn) - 1u);
    return __brev((s - 1u) >> 1) >> (32 - logn);
}

// modulus as doubles for the FP64 butterflies (moduli below 2^50 only; q = 0 otherwise)
struct FpQ {
    double q, qinv;       // modulus and 1/q as doubles; q = 0 where the modulus is too large for the FP64 paths
    double rinv, rinvq;   // 2^-64 mod q and that over q: takes a product with a multiplier-form operand back
};

// ---- context -----------------------------------------------------------------------------
#define CM_MAX_LIMBS 64
#define CM_MAX_DIGITS 16
#define CM_GAUSS_K 19
#define CM_KS_BATCH 8      // hoisted rotations whose ModDown runs as one batch
#define CM_NTT_MAX_LIMBS 1024

struct ConvTable {            // fast base conversion src -> dst (all indices into the modulus list)
    int ns = 0, nt = 0;
    std::vector<u64> inv_hat;     // [ns]   (hat_m^{-1} mod q_m), plain
    std::vector<u64> inv_hat_sh;  // [ns]   Shoup companion
    std::vector<u64> hat_mont;    // [ns*nt] (hat_m mod r) 2^64 mod r
    std::vector<int> src, dst;
};

// The same table in the form the conversion kernel reads (one per digit / per direction).
#define CONV_MAX_SRC 8
#define CONV_MAX_DST 64
struct ConvDev {
    int ns, nt;
    int src_mod[CONV_MAX_SRC], in_rows[CONV_MAX_SRC];
    u64 inv_hat[CONV_MAX_SRC], inv_hat_sh[CONV_MAX_SRC];
    int dst_mod[CONV_MAX_DST], out_rows[CONV_MAX_DST];
    u64 src_q[CONV_MAX_SRC], dst_q[CONV_MAX_DST], dst_qinv[CONV_MAX_DST];   // moduli and q^{-1} mod 2^64 inline
    u64 hat_mont[CONV_MAX_SRC * CONV_MAX_DST];      // [m * nt + r]
};

// per-kernel-family timing with HIP events on the launching stream (off unless enabled)
struct ProfState {
    bool on = false;
    std::vector<hipEvent_t> pool;
    struct Rec { int fam; double units; size_t e0; };
    std::vector<Rec> recs;
};

struct cm_ctx {
    cm_params prm;
    ProfState prof;
    int n, logn, L, K, alpha, nmod;      // nmod = L+1+K
    std::vector<u64> mod;                 // host copy of moduli
    std::vector<u64> psi;
    // device tables, indexed by modulus index
    ModC *d_modc = nullptr;               // [nmod]
    u64 *d_pmont = nullptr;               // [L+1] P = p_0 .. p_{K-1} mod q_i, multiplier (Montgomery) form
    u64 *d_ubound = nullptr;              // [nmod] q * floor(2^64 / q): uniform draws at or above it are rejected
    u64 *d_tw = nullptr, *d_twp = nullptr;      // forward twiddles psi^brev(i) and companions [nmod][n]
    u64 *d_itw = nullptr, *d_itwp = nullptr;    // inverse
    u64 *d_ninv = nullptr, *d_ninvp = nullptr;  // n^{-1} [nmod]
    // the same tables as doubles (w and w/q) for the limbs whose modulus is below 2^50
    FpQ *d_fpq = nullptr;                       // [nmod] (q, 1/q), q = 0 for larger moduli
    double *d_twd = nullptr, *d_twqd = nullptr, *d_itwd = nullptr, *d_itwqd = nullptr;
    double *d_ninvd = nullptr, *d_ninvqd = nullptr;
    std::vector<ModC> modc;
    // per-level tables (built lazily, kept): ModUp per digit, ModDown, rescale constants
    std::map<int, std::vector<ConvTable>> modup;   // level -> digit tables
    std::map<int, ConvTable> moddown;              // level -> P -> q_0..q_level
    std::map<int, u64 *> pinv;                     // level -> [level+1][2]: P^{-1} mod q_i, Shoup
    std::map<int, u64 *> qlinv;                    // level -> [level][2]: q_level^{-1} mod q_i, Shoup
    u64 *d_cdt = nullptr;                          // Gaussian table [CM_GAUSS_K]
    u64 cdt[CM_GAUSS_K];
    int lazy_terms;                                // products that may be summed before one REDC
    // options (cm_ctx_set_option)
    bool evk_stored_a = false;     // evaluation keys carry both halves; the inner products read the uniform half
    bool two_step_masks = false;   // cache appends multiply, store and rescale instead of fusing the product into the rescale
    // scratch arena
    u64 *arena = nullptr;
    size_t arena_words = 0;
    int *d_idx = nullptr;                          // 0, 1, 2, ...: modulus index lists of consecutive limbs
    int *d_idx_stage = nullptr;                    // [CM_NTT_MAX_LIMBS] staging of a caller's modulus index list (cm_ntt)
    // encode tables (host)
    std::vector<int> slot_pos;
    std::vector<double> tw_re, tw_im;              // omega^k
};

struct cm_sk {
    std::vector<int8_t> coeffs;
    u64 *d_ntt = nullptr;          // [nmod][n], Montgomery form, evaluation domain
    u64 noise = 0;                 // XORed into the public seed of a call to key its error streams
};

struct EvkEntry {
    u64 *d = nullptr;              // b halves [digits][nmod][n] (multiplier form, evaluation domain), then the
                                   // [digits][nmod] generator keys of the streams of the a halves (padded to an even
                                   // count), then -- stored_a only -- the a halves [digits][nmod][n] in multiplier form
};
struct cm_evk {
    int digits;
    bool stored_a = false;         // the option the set was generated under
    u64 seed = 0;                  // the (public) seed every key of the set was generated from
    std::map<u64, EvkEntry> keys;  // Galois element (0 = relinearisation)
};
// word offset of the stored a halves inside a key
inline size_t evk_a_offset(const cm_ctx *ctx) {
    const size_t digits = (size_t)(ctx->L + ctx->alpha) / ctx->alpha, nm = (size_t)ctx->nmod;
    return digits * nm * ctx->n + ((digits * nm + 1) & ~(size_t)1);
}

#define HIPCHK(x)                                  \
    do {                                           \
        hipError_t e_ = (x);                       \
        if (e_ != hipSuccess) {                    \
            cm_set_hip_error((int)e_);             \
            return CM_E_HIP;                       \
        }                                          \
    } while (0)
// Kernel launches report a bad configuration only through the runtime's last-error slot: the hot
// entry points end with this check (no synchronisation).
#define RETURN_LAUNCH_STATUS()                     \
    do {                                           \
        hipError_t e_ = hipPeekAtLastError();      \
        if (e_ != hipSuccess) {                    \
            cm_set_hip_error((int)e_);             \
            return CM_E_HIP;                       \
        }                                          \
        return CM_OK;                              \
    } while (0)
#define CMCHK(x)                \
    do {                        \
        cm_status s_ = (x);     \
        if (s_ != CM_OK) return s_; \
    } while (0)

void cm_set_hip_error(int e);
// Every extern "C" body that can reach an allocation (std::vector, std::map, new) sits between these: no C++
// exception crosses the boundary.
#define CM_TRY try {
#define CM_CATCH                                        \
    }                                                   \
    catch (const std::bad_alloc &) { return CM_E_NOMEM; } \
    catch (...) { return CM_E_INVAL; }

struct Prof {
    cm_ctx *c;
    hipStream_t st;
    size_t e0;
    bool live;
    Prof(cm_ctx *ctx, int fam, double units, hipStream_t st);
    ~Prof();
};

// ---- host helpers (context.hip) ------------------------------------------------------------
u64 h_mulmod(u64 a, u64 b, u64 q);
u64 h_powmod(u64 b, u64 e, u64 q);
u64 h_invmod(u64 a, u64 q);
u64 h_shoup(u64 w, u64 q);
u64 galois_of_step(const cm_ctx *ctx, int step);
const std::vector<ConvTable> &get_modup(cm_ctx *ctx, int level);
const ConvTable &get_moddown(cm_ctx *ctx, int level);
const u64 *get_pinv(cm_ctx *ctx, int level);
const u64 *get_qlinv(cm_ctx *ctx, int level);
std::vector<std::vector<int>> digits_at(const cm_ctx *ctx, int level);

// ---- kernel launchers ----------------------------------------------------------------------
// ntt.hip: limbs of n words each, limb i under modulus d_mod_idx[i] (device int array)
void launch_ntt(cm_ctx *ctx, u64 *data, const int *d_mod_idx, int limbs, bool inverse, hipStream_t st);
// convenience: limbs use consecutive modulus indices first, first+1, ...
void launch_ntt_range(cm_ctx *ctx, u64 *data, int first_mod, int limbs, bool inverse, hipStream_t st);
const int *iota_idx(cm_ctx *ctx);   // device array 0,1,2,...,CM_MAX_LIMBS-1
