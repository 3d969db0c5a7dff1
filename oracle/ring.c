/*
 * Oracle ring primitives -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, single-purpose C for the residue-number-system polynomial ring
 * Z_q[X]/(X^n + 1) that full-RNS CKKS works in (paper Sec. 2.1).  Every routine is
 * the textbook definition written out with `unsigned __int128` arithmetic; no
 * Montgomery/Barrett/Shoup forms, no lazy reduction, no blocking.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may load this library.
 *
 * Layout everywhere: a polynomial is `limbs` rows of `n` uint64 residues,
 * row i reduced modulo q[i], values in [0, q[i]).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef unsigned __int128 u128;

static inline u64 mulmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a * b) % q); }
static inline u64 addmod(u64 a, u64 b, u64 q) { u64 s = a + b; return s >= q ? s - q : s; }
static inline u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

static u64 powmod(u64 b, u64 e, u64 q) {
    u64 r = 1 % q;
    b %= q;
    while (e) {
        if (e & 1) r = mulmod(r, b, q);
        b = mulmod(b, b, q);
        e >>= 1;
    }
    return r;
}

u64 orc_mulmod(u64 a, u64 b, u64 q) { return mulmod(a, b, q); }
u64 orc_powmod(u64 b, u64 e, u64 q) { return powmod(b, e, q); }

/* Cyclic radix-2 transform of length n with root w (w^n = 1): bit-reverse the
 * input, then log2(n) rounds of butterflies.  out[k] = sum_i a[i] w^(ik). */
static void cyclic_dft(u64 *a, int n, u64 w, u64 q) {
    int logn = 0;
    while ((1 << logn) < n) logn++;
    for (int i = 0; i < n; i++) {
        int r = 0;
        for (int b = 0; b < logn; b++) if (i >> b & 1) r |= 1 << (logn - 1 - b);
        if (r > i) { u64 t = a[i]; a[i] = a[r]; a[r] = t; }
    }
    for (int len = 2; len <= n; len <<= 1) {
        u64 wl = powmod(w, (u64)(n / len), q);
        for (int s = 0; s < n; s += len) {
            u64 x = 1;
            for (int j = 0; j < len / 2; j++) {
                u64 u = a[s + j], v = mulmod(a[s + j + len / 2], x, q);
                a[s + j] = addmod(u, v, q);
                a[s + j + len / 2] = submod(u, v, q);
                x = mulmod(x, wl, q);
            }
        }
    }
}

/* Forward negacyclic transform, natural order in and out:
 *   out[k] = a(psi^(2k+1)) = sum_i a[i] psi^(i(2k+1)),   psi a primitive 2n-th root mod q.
 * Done as: twist by psi^i, then the cyclic transform with root psi^2. */
void orc_ntt(u64 *a, int limbs, int n, const u64 *q, const u64 *psi) {
#pragma omp parallel for schedule(dynamic)
    for (int l = 0; l < limbs; l++) {
        u64 *p = a + (size_t)l * n, x = 1;
        for (int i = 0; i < n; i++) { p[i] = mulmod(p[i], x, q[l]); x = mulmod(x, psi[l], q[l]); }
        cyclic_dft(p, n, mulmod(psi[l], psi[l], q[l]), q[l]);
    }
}

/* Inverse of orc_ntt. */
void orc_intt(u64 *a, int limbs, int n, const u64 *q, const u64 *psi) {
#pragma omp parallel for schedule(dynamic)
    for (int l = 0; l < limbs; l++) {
        u64 *p = a + (size_t)l * n, ql = q[l];
        u64 psi_inv = powmod(psi[l], ql - 2, ql);
        u64 n_inv = powmod((u64)n, ql - 2, ql);
        cyclic_dft(p, n, mulmod(psi_inv, psi_inv, ql), ql);
        u64 x = n_inv;
        for (int i = 0; i < n; i++) { p[i] = mulmod(p[i], x, ql); x = mulmod(x, psi_inv, ql); }
    }
}

/* out = a (op) b, coefficient-wise, per limb. */
void orc_add(u64 *out, const u64 *a, const u64 *b, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t k = (size_t)l * n + i;
            out[k] = addmod(a[k], b[k], q[l]);
        }
}
void orc_sub(u64 *out, const u64 *a, const u64 *b, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t k = (size_t)l * n + i;
            out[k] = submod(a[k], b[k], q[l]);
        }
}
void orc_mul(u64 *out, const u64 *a, const u64 *b, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t k = (size_t)l * n + i;
            out[k] = mulmod(a[k], b[k], q[l]);
        }
}
/* acc += a * b */
void orc_mac(u64 *acc, const u64 *a, const u64 *b, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t k = (size_t)l * n + i;
            acc[k] = addmod(acc[k], mulmod(a[k], b[k], q[l]), q[l]);
        }
}
/* out = a * c[l] with one scalar per limb */
void orc_mul_scalar(u64 *out, const u64 *a, const u64 *c, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t k = (size_t)l * n + i;
            out[k] = mulmod(a[k], c[l] % q[l], q[l]);
        }
}

/* Galois map a(X) -> a(X^g) on coefficient-domain limbs, g odd:
 * the monomial a_i X^i goes to a_i X^(ig mod 2n), and X^n = -1. */
void orc_automorphism(u64 *out, const u64 *a, int limbs, int n, const u64 *q, u64 g) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            u64 e = ((u64)i * g) % (2 * (u64)n);
            u64 v = a[(size_t)l * n + i];
            if (e < (u64)n) out[(size_t)l * n + e] = v;
            else out[(size_t)l * n + (e - n)] = v ? q[l] - v : 0;
        }
}

/* Signed integer coefficients -> residues. */
void orc_reduce_i64(u64 *out, const int64_t *c, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) {
            int64_t v = c[i] % (int64_t)q[l];
            out[(size_t)l * n + i] = v < 0 ? (u64)(v + (int64_t)q[l]) : (u64)v;
        }
}

/* Residues of one limb (representatives in [0, q_src)) re-reduced under other moduli. */
void orc_reduce_u64(u64 *out, const u64 *a, int limbs, int n, const u64 *q) {
#pragma omp parallel for
    for (int l = 0; l < limbs; l++)
        for (int i = 0; i < n; i++) out[(size_t)l * n + i] = a[i] % q[l];
}

/* Fast (approximate, non-centred, uncorrected) base conversion, coefficient domain:
 *   y_m   = a_m * inv_hat[m] mod qs[m]                      (in [0, qs[m]))
 *   out_r = sum_m y_m * hat_mod[m*nt + r]  mod qt[r]
 * where for source basis B = prod qs, hat_m = B/qs[m], inv_hat[m] = hat_m^{-1} mod qs[m],
 * hat_mod[m][r] = hat_m mod qt[r].  The integer represented is a + e*B with 0 <= e < ns. */
void orc_base_conv(u64 *out, const u64 *a, int ns, int nt, int n, const u64 *qs, const u64 *qt,
                   const u64 *inv_hat, const u64 *hat_mod) {
#pragma omp parallel for
    for (int r = 0; r < nt; r++)
        for (int i = 0; i < n; i++) {
            u64 acc = 0;
            for (int m = 0; m < ns; m++) {
                u64 y = mulmod(a[(size_t)m * n + i], inv_hat[m], qs[m]);
                acc = addmod(acc, mulmod(y % qt[r], hat_mod[(size_t)m * nt + r], qt[r]), qt[r]);
            }
            out[(size_t)r * n + i] = acc;
        }
}

/* ---- counter-based random numbers (integer only) --------------------------------
 * mix() is the SplitMix64 output function.  A draw is addressed by (seed, stream, ctr):
 *   key  = mix(mix(seed) ^ stream),  draw = mix(key + (ctr + 1) * GOLD).                */
#define GOLD 0x9E3779B97F4A7C15ULL
static inline u64 mix(u64 z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
static inline u64 draw(u64 key, u64 ctr) { return mix(key + (ctr + 1) * GOLD); }
u64 orc_rng_key(u64 seed, u64 stream) { return mix(mix(seed) ^ stream); }
u64 orc_rng_draw(u64 seed, u64 stream, u64 ctr) { return draw(orc_rng_key(seed, stream), ctr); }

/* Uniform residues: element i takes draws ctr = (attempt << 32) | i, attempt = 0,1,..,
 * and keeps the first one below q*floor(2^64/q), reduced mod q. */
void orc_sample_uniform(u64 *out, int n, u64 q, u64 seed, u64 stream) {
    u64 key = orc_rng_key(seed, stream);
    u64 bound = q * (u64)((((u128)1) << 64) / q);
    for (int i = 0; i < n; i++) {
        u64 att = 0, v;
        do { v = draw(key, (att << 32) | (u64)i); att++; } while (v >= bound);
        out[i] = v % q;
    }
}

/* Discrete Gaussian by cumulative table: element i takes one draw v; magnitude = number of
 * table entries cdt[k] (k < ncdt) with (v >> 1) >= cdt[k]; sign = lowest bit of v. */
void orc_sample_gauss(int64_t *out, int n, const u64 *cdt, int ncdt, u64 seed, u64 stream) {
    u64 key = orc_rng_key(seed, stream);
    for (int i = 0; i < n; i++) {
        u64 v = draw(key, (u64)i), u = v >> 1;
        int64_t mag = 0;
        for (int k = 0; k < ncdt; k++) mag += (u >= cdt[k]);
        out[i] = (v & 1) ? -mag : mag;
    }
}
