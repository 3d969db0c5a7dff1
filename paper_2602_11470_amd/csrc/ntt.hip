// Batched negacyclic NTT / inverse NTT over RNS limbs for gfx950.
//
// Transform: a(X) in Z_q[X]/(X^n+1)  ->  values a(psi^(2 brev(i)+1)) at position i (bit-reversed
// evaluation order), the merged-twiddle Cooley-Tukey / Gentleman-Sande pair.
//
// Decomposition for the 64-wide machine: n = 256 * n2.  A workgroup of 256 lanes owns 4096
// words; every lane keeps 16 of them in registers and runs four butterfly stages there
// (radix 16), then the workgroup transposes through LDS and runs four more.
//   column kernel : stages 0..7, a tile of 256 rows x 16 adjacent columns (rows n2 apart)
//   row kernel    : the remaining log2(n2) stages on contiguous blocks of n2 words
// so a limb makes two round trips to HBM for n = 65536 (and for n = 4096).
//
// Two butterfly arithmetics, chosen per limb (uniform per workgroup):
//   IntArith : Harvey's lazy butterflies with Shoup twiddles on u64 (any modulus below 2^62);
//              ~32 VALU instructions per butterfly on this machine.
//   FpArith  : for moduli below 2^50, residues held as exact integers in doubles.  FP64 FMA
//              issues at full rate here, and a modular product is 6 instructions:
//                  h = y*w; l = fma(y, w, -h)            (exact product h + l)
//                  c = rint(y * (w/q)); r = fma(-c, q, h) + l
//              exact because |h - c q| < 2^53 whenever |y| <= 2.1 q; r = y w (mod q), |r| <= 1.04 q.
//              Values stay signed and lazy (|v| <= 1.54 q), one 3-instruction renormalisation per
//              butterfly; ~11 instructions per butterfly.  Between the two kernels of a
//              transform the words in memory are raw doubles; at rest they are u64 in [0, q).
// Both give bit-identical results (all steps are exact integer arithmetic).
#include "kernels.h"

#define NTT_THREADS 256

struct NttTables {
    const ModC *modc;
    const u64 *tw, *twp;          // [nmod][n] integer twiddles and Shoup companions
    const double *twd, *twqd;     // [nmod][n] the same twiddles as doubles, and w/q
    const u64 *ninv, *ninvp;      // [nmod] n^{-1} (inverse only)
    const double *ninvd, *ninvqd;
    const FpQ *fpq;               // [nmod] q and 1/q as doubles; q = 0 where the limb must use IntArith
    // Large launches (256 limbs and more) read with non-temporal loads: their input was written long before and is read
    // once.  Small launches find theirs in the caches and read plainly (a single key switch is 3 % slower otherwise).
    int stream_loads;
};

// ---- integer arithmetic --------------------------------------------------------------------------
struct IntArith {
    typedef u64 T;
    u64 q, q2, ni, nip;
    const u64 *w, *wp;
    __device__ __forceinline__ void init(const NttTables &t, int mi, int n) {
        q = t.modc[mi].q, q2 = 2 * q;
        w = t.tw + (size_t)mi * n, wp = t.twp + (size_t)mi * n;
        ni = nip = 0;
        if (t.ninv) ni = t.ninv[mi], nip = t.ninvp[mi];
    }
    __device__ __forceinline__ T from_rest(u64 raw) const { return raw; }     // canonical [0, q)
    __device__ __forceinline__ T from_mid(u64 raw) const { return raw; }
    __device__ __forceinline__ u64 to_mid(T v) const { return v; }
    typedef u64 W;
    __device__ __forceinline__ void load_tw(u64 idx, W &a, W &b) const { a = w[idx], b = wp[idx]; }
    __device__ __forceinline__ void ct(T &X, T &Y, W a, W b) const {           // in, out below 4q
        u64 x = X >= q2 ? X - q2 : X;
        u64 t = mul_shoup_lazy(Y, a, b, q);
        X = x + t;
        Y = x - t + q2;
    }
    __device__ __forceinline__ void gs(T &X, T &Y, W a, W b) const {           // in, out below 2q
        u64 s = X + Y, d = X - Y + q2;
        X = s >= q2 ? s - q2 : s;
        Y = mul_shoup_lazy(d, a, b, q);
    }
    __device__ __forceinline__ u64 to_rest_fwd(T v) const {
        v = v >= q2 ? v - q2 : v;
        return v >= q ? v - q : v;
    }
    __device__ __forceinline__ u64 to_rest_inv(T v) const { return mul_shoup(v, ni, nip, q); }
};

// ---- FP64 arithmetic for moduli below 2^50 -----------------------------------------------------------
#define TWO52 4503599627370496.0
struct FpArith {
    typedef double T;
    double q, qinv, ni, niq;
    const double *w, *wq;
    __device__ __forceinline__ void init(const NttTables &t, int mi, int n) {
        q = t.fpq[mi].q, qinv = t.fpq[mi].qinv;
        w = t.twd + (size_t)mi * n, wq = t.twqd + (size_t)mi * n;
        ni = niq = 0.0;
        if (t.ninvd) ni = t.ninvd[mi], niq = t.ninvqd[mi];
    }
    __device__ __forceinline__ double mulmod(double y, double a, double aq) const {
        double h = y * a;
        double l = __builtin_fma(y, a, -h);
        double c = __builtin_rint(y * aq);
        return __builtin_fma(-c, q, h) + l;
    }
    __device__ __forceinline__ double norm(double x) const { return __builtin_fma(-__builtin_rint(x * qinv), q, x); }
    __device__ __forceinline__ T from_rest(u64 raw) const {
        return __longlong_as_double((long long)(raw | 0x4330000000000000ULL)) - TWO52;
    }
    __device__ __forceinline__ T from_mid(u64 raw) const { return __longlong_as_double((long long)raw); }
    __device__ __forceinline__ u64 to_mid(T v) const { return (u64)__double_as_longlong(v); }
    typedef double W;
    __device__ __forceinline__ void load_tw(u64 idx, W &a, W &b) const { a = w[idx], b = wq[idx]; }
    // With table twiddles (0 <= w < q, w/q correctly rounded) |r| <= 1.04 q; with generated ones
    // (|w| <= 0.9 q, w/q taken as w * (1/q)) |r| <= 1.2 q.  Either way every value stays below 2.1 q.
    __device__ __forceinline__ void ct(T &X, T &Y, W a, W b) const {
        double x = norm(X), r = mulmod(Y, a, b);
        X = x + r;
        Y = x - r;
    }
    __device__ __forceinline__ void gs(T &X, T &Y, W a, W b) const {
        double s = X + Y, d = X - Y;
        X = norm(s);
        Y = mulmod(d, a, b);
    }
    __device__ __forceinline__ u64 canon(double v) const {                     // |v| < 2^52  ->  [0, q)
        double r = __builtin_fma(-__builtin_floor(v * qinv), q, v);
        r = r < 0.0 ? r + q : r;
        r = r >= q ? r - q : r;
        return (u64)__double_as_longlong(r + TWO52) & 0x000FFFFFFFFFFFFFULL;
    }
    __device__ __forceinline__ u64 to_rest_fwd(T v) const { return canon(v); }
    __device__ __forceinline__ u64 to_rest_inv(T v) const { return canon(mulmod(v, ni, niq)); }
};

// Twiddle providers for four stages starting at stage s0 with base0 = 2^s0 + (block index):
// stage s0 + a, group g uses table entry (base0 << a) + g.
// Integer limbs read the entry and its companion where the butterfly uses them.  FP64 limbs read all fifteen
// entries up front (one exposure to memory latency instead of one per stage, and the loads overlap the data loads
// or the LDS exchange in front of them); the second factor w/q is taken as w * (1/q), one multiplication instead
// of a second table: the quotient estimate may then be off by one more unit, the product stays exact
// (|r| <= 1.3 q for |y| <= 2.1 q).
template <class A>
struct TableTw;
template <>
struct TableTw<IntArith> {
    const IntArith &ar;
    u64 base0;
    __device__ __forceinline__ TableTw(const IntArith &a_, u64 b0) : ar(a_), base0(b0) {}
    __device__ __forceinline__ void get(int a, int g, u64 &w0, u64 &w1) const { ar.load_tw((base0 << a) + g, w0, w1); }
};
template <>
struct TableTw<FpArith> {
    const FpArith &ar;
    double w[15];
    __device__ __forceinline__ TableTw(const FpArith &a_, u64 b0) : ar(a_) {
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int g = 0; g < (1 << a); g++) w[(1 << a) - 1 + g] = ar.w[(b0 << a) + g];
    }
    __device__ __forceinline__ void get(int a, int g, double &w0, double &w1) const {
        w0 = w[(1 << a) - 1 + g];
        w1 = w0 * ar.qinv;
    }
};
// The same entries computed from ONE table word (FP64 limbs): with T_a = tw[base0 << a],
//   T_2 = T_3^2, T_1 = T_2^2, T_0 = T_1^2      (the exponent brev(base0) >> a doubles each time)
//   tw[(base0 << a) + g] = T_a * tw[g]          (the low bits g reverse into the top of the exponent)
// which removes almost all twiddle traffic of the last four stages, where every lane has its own 15.
struct GenTw {
    const FpArith &ar;
    double T[4];
    __device__ __forceinline__ GenTw(const FpArith &a_, u64 base0) : ar(a_) {
        T[3] = ar.w[base0 << 3];
        T[2] = ar.mulmod(T[3], T[3], T[3] * ar.qinv);
        T[1] = ar.mulmod(T[2], T[2], T[2] * ar.qinv);
        T[0] = ar.mulmod(T[1], T[1], T[1] * ar.qinv);
    }
    __device__ __forceinline__ void get(int a, int g, double &w0, double &w1) const {
        w0 = g ? ar.mulmod(T[a], ar.w[g], ar.wq[g]) : T[a];
        w1 = w0 * ar.qinv;
    }
};

// Four forward stages on 16 register values whose index k is the local position inside one
// butterfly block of the first of these stages.
template <class A, class TW>
__device__ __forceinline__ void radix16_fwd_tw(typename A::T (&v)[16], const A &ar, const TW &tw) {
#pragma unroll
    for (int a = 0; a < 4; a++) {
        const int half = 8 >> a;
#pragma unroll
        for (int g = 0; g < (1 << a); g++) {
            typename A::W w0, w1;
            tw.get(a, g, w0, w1);
#pragma unroll
            for (int j = 0; j < half; j++) {
                int k = g * 2 * half + j;
                ar.ct(v[k], v[k + half], w0, w1);
            }
        }
    }
}
// The inverse of the above (stages in the opposite order).
template <class A, class TW>
__device__ __forceinline__ void radix16_inv_tw(typename A::T (&v)[16], const A &ar, const TW &tw) {
#pragma unroll
    for (int a = 3; a >= 0; a--) {
        const int half = 8 >> a;
#pragma unroll
        for (int g = 0; g < (1 << a); g++) {
            typename A::W w0, w1;
            tw.get(a, g, w0, w1);
#pragma unroll
            for (int j = 0; j < half; j++) {
                int k = g * 2 * half + j;
                ar.gs(v[k], v[k + half], w0, w1);
            }
        }
    }
}
// last four stages of the row pass: generated twiddles for FP64 limbs, table for the others
__device__ __forceinline__ void radix16_fwd_last(double (&v)[16], const FpArith &ar, u64 base0) {
    radix16_fwd_tw(v, ar, GenTw(ar, base0));
}
__device__ __forceinline__ void radix16_fwd_last(u64 (&v)[16], const IntArith &ar, u64 base0) {
    radix16_fwd_tw(v, ar, TableTw<IntArith>(ar, base0));
}
__device__ __forceinline__ void radix16_inv_last(double (&v)[16], const FpArith &ar, u64 base0) {
    radix16_inv_tw(v, ar, GenTw(ar, base0));
}
__device__ __forceinline__ void radix16_inv_last(u64 (&v)[16], const IntArith &ar, u64 base0) {
    radix16_inv_tw(v, ar, TableTw<IntArith>(ar, base0));
}

// LDS index with one pad word per 16 so that lanes reading words 16 apart hit distinct banks
// The passes write with non-temporal stores: a limb is read again only by a later kernel, after hundreds of MiB of other
// limbs have gone by (measured: 1 % off the transforms of a step against plain stores).
#define NTT_ST(ptr, val) __builtin_nontemporal_store((u64)(val), (ptr))
// the masked products of a cache append read the cached ciphertext they add to and write it back past the caches (the
// cache is gigabytes; 3 % off an append)
#define TAIL_LD(ptr) __builtin_nontemporal_load(ptr)
#define TAIL_ST(ptr, val) __builtin_nontemporal_store((u64)(val), (ptr))
__device__ __forceinline__ int pad(int e) { return e + (e >> 4); }
#define LDS_WORDS (4096 + 256)

// ---- column passes: stages 0..7; tile = rows 0..255 of 16 adjacent columns ---------------------------
template <class A>
__device__ __forceinline__ void cols_fwd_body(u64 *lds, u64 *p, const u64 *ps, const NttTables &t, int mi, int n, int n2) {
    A ar;
    ar.init(t, mi, n);
    const int c = threadIdx.x & 15, sub = threadIdx.x >> 4;
    typename A::T v[16];
    u64 raw[16];
    if (t.stream_loads) {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = __builtin_nontemporal_load(ps + (unsigned)((sub + 16 * k) * n2 + c));
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = ps[(unsigned)((sub + 16 * k) * n2 + c)];
    }
    {
        const TableTw<A> tw(ar, 1);                 // in flight together with the data
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = ar.from_rest(raw[k]);
        radix16_fwd_tw(v, ar, tw);
    }
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad((sub + 16 * k) * 16 + c)] = ar.to_mid(v[k]);
    const TableTw<A> tw2(ar, 16 + sub);             // in flight across the exchange
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ar.from_mid(lds[pad((16 * sub + k) * 16 + c)]);
    radix16_fwd_tw(v, ar, tw2);
#pragma unroll
    for (int k = 0; k < 16; k++) NTT_ST(p + (unsigned)((16 * sub + k) * n2 + c), ar.to_mid(v[k]));
}
template <class A>
__device__ __forceinline__ void cols_inv_body(u64 *lds, u64 *p, const NttTables &t, int mi, int n, int n2) {
    A ar;
    ar.init(t, mi, n);
    const int c = threadIdx.x & 15, sub = threadIdx.x >> 4;
    typename A::T v[16];
    u64 raw[16];
    if (t.stream_loads) {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = __builtin_nontemporal_load(p + (unsigned)((16 * sub + k) * n2 + c));
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = p[(unsigned)((16 * sub + k) * n2 + c)];
    }
    {
        const TableTw<A> tw(ar, 16 + sub);          // in flight together with the data
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = ar.from_mid(raw[k]);
        radix16_inv_tw(v, ar, tw);
    }
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad((16 * sub + k) * 16 + c)] = ar.to_mid(v[k]);
    const TableTw<A> tw2(ar, 1);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ar.from_mid(lds[pad((sub + 16 * k) * 16 + c)]);
    radix16_inv_tw(v, ar, tw2);
#pragma unroll
    for (int k = 0; k < 16; k++) NTT_ST(p + (unsigned)((sub + 16 * k) * n2 + c), ar.to_rest_inv(v[k]));
}

// grid.x = limbs * (n2/16)
__global__ __launch_bounds__(NTT_THREADS) void ntt_cols_fwd(u64 *__restrict__ data, const u64 *__restrict__ src,
                                                           const int *__restrict__ src_rows,
                                                           const int *__restrict__ rows,
                                                           const int *__restrict__ mod_idx, NttTables t, int n,
                                                           int n2) {
    __shared__ u64 lds[LDS_WORDS];
    const int tiles = n2 >> 4;
    const int limb = blockIdx.x / tiles, c0 = (blockIdx.x % tiles) << 4;
    const int mi = mod_idx[limb];
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + c0;
    const u64 *ps = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n + c0 : p;
    if (t.fpq[mi].q != 0.0)
        cols_fwd_body<FpArith>(lds, p, ps, t, mi, n, n2);
    else
        cols_fwd_body<IntArith>(lds, p, ps, t, mi, n, n2);
}
__global__ __launch_bounds__(NTT_THREADS) void ntt_cols_inv(u64 *__restrict__ data, const int *__restrict__ rows,
                                                           const int *__restrict__ mod_idx, NttTables t, int n,
                                                           int n2) {
    __shared__ u64 lds[LDS_WORDS];
    const int tiles = n2 >> 4;
    const int limb = blockIdx.x / tiles, c0 = (blockIdx.x % tiles) << 4;
    const int mi = mod_idx[limb];
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + c0;
    if (t.fpq[mi].q != 0.0)
        cols_inv_body<FpArith>(lds, p, t, mi, n, n2);
    else
        cols_inv_body<IntArith>(lds, p, t, mi, n, n2);
}

// ---- 16 x 16 transpose inside a row of 16 lanes, by cross-lane moves instead of a trip through LDS -----------------
// lane s, register k  <->  lane k, register s: four exchange stages with the partner lane s ^ b (b = 8, 4, 2, 1); in the
// stage of b the pair of registers (k, k | b) trades one member with the partner.  b = 8 and 4 are DPP row moves that
// write only the banks (groups of four lanes) on one side; b = 2 and 1 are quad permutations with selects around them:
// 96 DPP moves and 96 selects per lane.  The row passes use it for the exchange between their two radix-16 groups
// (the sixteen lanes that share a block of 256 words); measured against the LDS exchange it replaces (32 LDS
// instructions and a barrier) it is time-neutral, within 2 % either way from 24 to 1008 limbs per launch.
template <int CTRL, int BANKS>
__device__ __forceinline__ u64 dpp_merge(u64 old, u64 src) {
    const int lo = __builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, 0xF, BANKS, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(old >> 32), (int)(src >> 32), CTRL, 0xF, BANKS, false);
    return ((u64)(unsigned)hi << 32) | (unsigned)lo;
}
template <int CTRL>
__device__ __forceinline__ u64 dpp_all(u64 src) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)src, CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(src >> 32), CTRL, 0xF, 0xF, false);
    return ((u64)(unsigned)hi << 32) | (unsigned)lo;
}
__device__ __forceinline__ void transpose16(u64 (&x)[16], int s) {
#pragma unroll
    for (int k = 0; k < 16; k++)
        if (!(k & 8)) {
            const u64 a = x[k], b = x[k | 8];
            x[k] = dpp_merge<0x128, 0xC>(a, b);          // lanes 8..15 take the partner's upper register (row_ror:8)
            x[k | 8] = dpp_merge<0x128, 0x3>(b, a);      // lanes 0..7 take the partner's lower register
        }
#pragma unroll
    for (int k = 0; k < 16; k++)
        if (!(k & 4)) {
            const u64 a = x[k], b = x[k | 4];
            x[k] = dpp_merge<0x114, 0xA>(a, b);          // row_shr:4 into the banks with bit 2 set
            x[k | 4] = dpp_merge<0x104, 0x5>(b, a);      // row_shl:4 into the others
        }
    const bool h2 = s & 2, h1 = s & 1;
#pragma unroll
    for (int k = 0; k < 16; k++)
        if (!(k & 2)) {
            const u64 a = x[k], b = x[k | 2];
            const u64 r = dpp_all<0x4E>(h2 ? a : b);     // quad_perm [2, 3, 0, 1]
            x[k] = h2 ? r : a, x[k | 2] = h2 ? b : r;
        }
#pragma unroll
    for (int k = 0; k < 16; k++)
        if (!(k & 1)) {
            const u64 a = x[k], b = x[k | 1];
            const u64 r = dpp_all<0xB1>(h1 ? a : b);     // quad_perm [1, 0, 3, 2]
            x[k] = h1 ? r : a, x[k | 1] = h1 ? b : r;
        }
}
template <class A>
__device__ __forceinline__ void transpose16(typename A::T (&v)[16], const A &ar, int s) {
    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = ar.to_mid(v[k]);
    transpose16(x, s);
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ar.from_mid(x[k]);
}

// ---- row passes on contiguous blocks of 256 words (n = 65536): a workgroup owns 16 blocks ---------------
template <class A, bool TAIL>
__device__ __forceinline__ void rows256_fwd_body(u64 *lds, u64 *p, const NttTables &t, int mi, int n, int chunk,
                                                 int limb, const FinishBatch &fb) {
    A ar;
    ar.init(t, mi, n);
    const int sub = threadIdx.x & 15, blk = threadIdx.x >> 4;
    const u64 B = (u64)chunk * 16 + blk;
    typename A::T v[16];
    u64 raw[16];
    if (t.stream_loads) {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = __builtin_nontemporal_load(p + blk * 256 + sub + 16 * k);
    } else {
#pragma unroll
        for (int k = 0; k < 16; k++) raw[k] = p[blk * 256 + sub + 16 * k];
    }
    {
        const TableTw<A> tw(ar, 256 + B);           // in flight together with the data
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = ar.from_mid(raw[k]);
        radix16_fwd_tw(v, ar, tw);
    }
    transpose16(v, ar, sub);           // word sub + 16 k of the block -> word 16 sub + k
    radix16_fwd_last(v, ar, 4096 + B * 16 + sub);
    // Each lane now owns 16 contiguous words.  A trip through LDS (the only one of this pass) hands every lane the
    // words tid, tid + 256, ... of the tile instead, so that all global traffic below is coalesced.
#pragma unroll
    for (int k = 0; k < 16; k++) lds[pad(blk * 256 + 16 * sub + k)] = ar.to_rest_fwd(v[k]);
    __syncthreads();
    if (!TAIL) {
#pragma unroll
        for (int k = 0; k < 16; k++) NTT_ST(p + threadIdx.x + 256 * k, lds[pad(threadIdx.x + 256 * k)]);
        return;
    }
    // fused ModDown tail: this limb is NTT(conv) of item r, component c, limb l
    const int per = fb.ncomp * (fb.level + 1);
    const int r = limb / per, c = fb.comp0 + (limb % per) / (fb.level + 1), l = limb % (fb.level + 1);
    const u64 q = t.modc[l].q, pi = fb.pinv[2 * l], pis = fb.pinv[2 * l + 1];
    const unsigned pos0 = (unsigned)chunk * 4096 + threadIdx.x;
    const size_t row = ((size_t)c * (fb.level + 1) + l) * n;
    const u64 *up = fb.u[r] + ((size_t)c * fb.ext + l) * n + pos0;
    const u64 *ad = (fb.addend[r] && c < fb.addend_comps) ? fb.addend[r] + row : nullptr;
    const u64 *ac = fb.accum[r] ? fb.accum[r] + row + pos0 : nullptr;
    u64 *op = fb.out[r] + row + pos0;
    const unsigned g = fb.g[r];
    const int logn = 31 - __clz(n);
    // All operands of the tail are loaded first, then combined: sixteen independent loads per stream are in flight at
    // once instead of one load-wait-use chain per word.
    u64 uu[16], aa[16], cc[16];
    if (fb.mul_pt) {
        // u = u[r] * (mul_pt through the Galois map mul_g[r]), formed here instead of being read
        const u64 qinv = t.modc[l].qinv;
        const u64 *mp = fb.mul_pt + (size_t)l * n;
        const unsigned mg = fb.mul_g[r];
#pragma unroll
        for (int k = 0; k < 16; k++) uu[k] = up[256 * k];
        if (mg) {
#pragma unroll
            for (int k = 0; k < 16; k++) aa[k] = mp[perm_src(pos0 + 256 * k, mg, logn)];
        } else {
#pragma unroll
            for (int k = 0; k < 16; k++) aa[k] = mp[pos0 + 256 * k];
        }
        if (ac) {
#pragma unroll
            for (int k = 0; k < 16; k++) cc[k] = TAIL_LD(ac + 256 * k);
        }
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const u64 uv = redc((u128)uu[k] * aa[k], q, qinv);
            u64 x = mul_shoup(submod(uv, lds[pad(threadIdx.x + 256 * k)], q), pi, pis, q);
            if (ac) x = addmod(x, cc[k], q);
            TAIL_ST(op + 256 * k, x);
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < 16; k++) uu[k] = up[256 * k];
    if (ad && g) {
#pragma unroll
        for (int k = 0; k < 16; k++) aa[k] = ad[perm_src(pos0 + 256 * k, g, logn)];
    } else if (ad) {
#pragma unroll
        for (int k = 0; k < 16; k++) aa[k] = ad[pos0 + 256 * k];
    }
    if (ac) {
#pragma unroll
        for (int k = 0; k < 16; k++) cc[k] = ac[256 * k];
    }
#pragma unroll
    for (int k = 0; k < 16; k++) {
        u64 d = submod(uu[k], lds[pad(threadIdx.x + 256 * k)], q);
        u64 x = mul_shoup(d, pi, pis, q);
        if (ad) x = addmod(x, aa[k], q);
        if (ac) x = addmod(x, cc[k], q);
        op[256 * k] = x;
    }
}
template <class A>
__device__ __forceinline__ void rows256_inv_body(u64 *lds, u64 *p, const u64 *ps, const u64 *psrow, unsigned g,
                                                 const NttTables &t, int mi, int n, int chunk) {
    A ar;
    ar.init(t, mi, n);
    const int sub = threadIdx.x & 15, blk = threadIdx.x >> 4;
    const u64 B = (u64)chunk * 16 + blk;
    typename A::T v[16];
    // coalesced load (through the Galois permutation if g != 0: a run of 64 positions maps onto one
    // aligned run of 64), then every lane picks its 16 contiguous words from LDS
    {
        const int logn = 31 - __clz(n);
        const unsigned pos0 = (unsigned)chunk * 4096 + threadIdx.x;
        u64 w[16];                        // sixteen independent loads in flight, then the writes to LDS
        if (g) {
#pragma unroll
            for (int k = 0; k < 16; k++) w[k] = psrow[perm_src(pos0 + 256 * k, g, logn)];
        } else if (t.stream_loads) {
#pragma unroll
            for (int k = 0; k < 16; k++) w[k] = __builtin_nontemporal_load(ps + threadIdx.x + 256 * k);
        } else {
#pragma unroll
            for (int k = 0; k < 16; k++) w[k] = ps[threadIdx.x + 256 * k];
        }
#pragma unroll
        for (int k = 0; k < 16; k++) lds[pad(threadIdx.x + 256 * k)] = w[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = ar.from_rest(lds[pad(blk * 256 + 16 * sub + k)]);
    }
    radix16_inv_last(v, ar, 4096 + B * 16 + sub);
    const TableTw<A> tw2(ar, 256 + B);
    transpose16(v, ar, sub);           // word 16 sub + k of the block -> word sub + 16 k
    radix16_inv_tw(v, ar, tw2);
#pragma unroll
    for (int k = 0; k < 16; k++) NTT_ST(p + blk * 256 + sub + 16 * k, ar.to_mid(v[k]));
}
// grid.x = limbs * n/4096; TAIL: the fused ModDown / rescale tail (a kernel of its own, so that the registers its
// operands take do not lower the occupancy of the plain transform)
template <bool TAIL>
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows256_fwd(u64 *__restrict__ data, const int *__restrict__ rows,
                                                              const int *__restrict__ mod_idx, NttTables t, int n,
                                                              FinishBatch fb) {
    __shared__ u64 lds[LDS_WORDS];
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + (size_t)chunk * 4096;
    if (t.fpq[mi].q != 0.0)
        rows256_fwd_body<FpArith, TAIL>(lds, p, t, mi, n, chunk, limb, fb);
    else
        rows256_fwd_body<IntArith, TAIL>(lds, p, t, mi, n, chunk, limb, fb);
}
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows256_inv(u64 *__restrict__ data, const u64 *__restrict__ src,
                                                              const int *__restrict__ src_rows,
                                                              const int *__restrict__ rows,
                                                              const int *__restrict__ mod_idx, NttTables t, int n,
                                                              unsigned g) {
    __shared__ u64 lds[LDS_WORDS];
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + (size_t)chunk * 4096;
    const u64 *psrow = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n : p - (size_t)chunk * 4096;
    const u64 *ps = psrow + (size_t)chunk * 4096;
    if (t.fpq[mi].q != 0.0)
        rows256_inv_body<FpArith>(lds, p, ps, psrow, g, t, mi, n, chunk);
    else
        rows256_inv_body<IntArith>(lds, p, ps, psrow, g, t, mi, n, chunk);
}

// ---- row passes on blocks of 16 words (n = 4096): every lane owns one block ---------------------------------
template <class A>
__device__ __forceinline__ void rows16_fwd_body(u64 *p, const NttTables &t, int mi, int n, u64 B) {
    A ar;
    ar.init(t, mi, n);
    typename A::T v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ar.from_mid(p[k]);
    radix16_fwd_tw(v, ar, TableTw<A>(ar, 256 + B));
#pragma unroll
    for (int k = 0; k < 16; k++) p[k] = ar.to_rest_fwd(v[k]);
}
template <class A>
__device__ __forceinline__ void rows16_inv_body(u64 *p, const u64 *ps, const u64 *psrow, unsigned g,
                                                const NttTables &t, int mi, int n, u64 B) {
    A ar;
    ar.init(t, mi, n);
    typename A::T v[16];
    const int logn = 31 - __clz(n);
#pragma unroll
    for (int k = 0; k < 16; k++)
        v[k] = ar.from_rest(g ? psrow[perm_src((unsigned)(B * 16 + k), g, logn)] : ps[k]);
    radix16_inv_tw(v, ar, TableTw<A>(ar, 256 + B));
#pragma unroll
    for (int k = 0; k < 16; k++) p[k] = ar.to_mid(v[k]);
}
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows16_fwd(u64 *__restrict__ data, const int *__restrict__ rows,
                                                             const int *__restrict__ mod_idx, NttTables t, int n) {
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 B = (u64)chunk * 256 + threadIdx.x;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + B * 16;
    if (t.fpq[mi].q != 0.0)
        rows16_fwd_body<FpArith>(p, t, mi, n, B);
    else
        rows16_fwd_body<IntArith>(p, t, mi, n, B);
}
__global__ __launch_bounds__(NTT_THREADS) void ntt_rows16_inv(u64 *__restrict__ data, const u64 *__restrict__ src,
                                                             const int *__restrict__ src_rows,
                                                             const int *__restrict__ rows,
                                                             const int *__restrict__ mod_idx, NttTables t, int n,
                                                             unsigned g) {
    const int per = n >> 12;
    const int limb = blockIdx.x / per, chunk = blockIdx.x % per;
    const int mi = mod_idx[limb];
    const u64 B = (u64)chunk * 256 + threadIdx.x;
    u64 *p = data + (size_t)(rows ? rows[limb] : limb) * n + B * 16;
    const u64 *psrow = src ? src + (size_t)(src_rows ? src_rows[limb] : limb) * n : p - B * 16;
    const u64 *ps = psrow + B * 16;
    if (t.fpq[mi].q != 0.0)
        rows16_inv_body<FpArith>(p, ps, psrow, g, t, mi, n, B);
    else
        rows16_inv_body<IntArith>(p, ps, psrow, g, t, mi, n, B);
}

// data rows d_rows[i] (or i) are transformed in place; with src != nullptr the first pass reads row
// src_rows[i] (or i) of src instead, so the transform is out of place and src is left untouched.
// With g != 0 (inverse, out of place only) the source is read through the Galois permutation, i.e.
// the result is the coefficient form of the mapped polynomial.
void launch_ntt_src(cm_ctx *ctx, u64 *data, const int *d_rows, const u64 *src, const int *d_src_rows,
                    const int *d_mod_idx, int limbs, bool inverse, hipStream_t st, u64 g) {
    if (limbs <= 0) return;
    if (g && (!inverse || !src || src == data)) g = 0;
    Prof prof_(ctx, inverse ? CM_K_NTT_INV : CM_K_NTT_FWD, limbs, st);
    const int n = ctx->n, n2 = n >> 8;
    dim3 grid((unsigned)limbs * (n >> 12)), block(NTT_THREADS);
    NttTables t;
    t.modc = ctx->d_modc, t.fpq = ctx->d_fpq;
    t.stream_loads = limbs >= 256;
    if (!inverse) {
        t.tw = ctx->d_tw, t.twp = ctx->d_twp, t.twd = ctx->d_twd, t.twqd = ctx->d_twqd;
        t.ninv = t.ninvp = nullptr, t.ninvd = t.ninvqd = nullptr;
        hipLaunchKernelGGL(ntt_cols_fwd, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx, t, n, n2);
        if (n2 == 256)
            hipLaunchKernelGGL(ntt_rows256_fwd<false>, grid, block, 0, st, data, d_rows, d_mod_idx, t, n, FinishBatch());
        else
            hipLaunchKernelGGL(ntt_rows16_fwd, grid, block, 0, st, data, d_rows, d_mod_idx, t, n);
    } else {
        t.tw = ctx->d_itw, t.twp = ctx->d_itwp, t.twd = ctx->d_itwd, t.twqd = ctx->d_itwqd;
        t.ninv = ctx->d_ninv, t.ninvp = ctx->d_ninvp, t.ninvd = ctx->d_ninvd, t.ninvqd = ctx->d_ninvqd;
        if (n2 == 256)
            hipLaunchKernelGGL(ntt_rows256_inv, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx, t, n,
                               (unsigned)g);
        else
            hipLaunchKernelGGL(ntt_rows16_inv, grid, block, 0, st, data, src, d_src_rows, d_rows, d_mod_idx, t, n,
                               (unsigned)g);
        hipLaunchKernelGGL(ntt_cols_inv, grid, block, 0, st, data, d_rows, d_mod_idx, t, n, n2);
    }
}
void launch_ntt_fwd_finish(cm_ctx *ctx, u64 *conv, const int *d_mods, const FinishBatch &fb, hipStream_t st, const u64 *src,
                           const int *d_src_rows) {
    const int limbs = fb.items * fb.ncomp * (fb.level + 1), n = ctx->n;
    if (limbs <= 0) return;
    Prof prof_(ctx, CM_K_NTT_FWD, limbs, st);
    dim3 grid((unsigned)limbs * (n >> 12)), block(NTT_THREADS);
    NttTables t;
    t.modc = ctx->d_modc, t.fpq = ctx->d_fpq;
    t.stream_loads = limbs >= 256;
    t.tw = ctx->d_tw, t.twp = ctx->d_twp, t.twd = ctx->d_twd, t.twqd = ctx->d_twqd;
    t.ninv = t.ninvp = nullptr, t.ninvd = t.ninvqd = nullptr;
    hipLaunchKernelGGL(ntt_cols_fwd, grid, block, 0, st, conv, src, d_src_rows, (const int *)nullptr, d_mods, t, n, n >> 8);
    hipLaunchKernelGGL(ntt_rows256_fwd<true>, grid, block, 0, st, conv, (const int *)nullptr, d_mods, t, n, fb);
}
void launch_ntt_rows(cm_ctx *ctx, u64 *data, const int *d_rows, const int *d_mod_idx, int limbs,
                     bool inverse, hipStream_t st) {
    launch_ntt_src(ctx, data, d_rows, nullptr, nullptr, d_mod_idx, limbs, inverse, st, 0);
}
void launch_ntt(cm_ctx *ctx, u64 *data, const int *d_mod_idx, int limbs, bool inverse,
                hipStream_t st) {
    launch_ntt_rows(ctx, data, nullptr, d_mod_idx, limbs, inverse, st);
}
void launch_ntt_range(cm_ctx *ctx, u64 *data, int first_mod, int limbs, bool inverse,
                      hipStream_t st) {
    launch_ntt(ctx, data, iota_idx(ctx) + first_mod, limbs, inverse, st);
}
