"""Oracle: plain CPU full-RNS CKKS (TEST INFRASTRUCTURE, not product code).

The paper treats the CKKS operations as given (Sec. 2.1: addition, ct-pt and ct-ct
multiplication, rotation, level drop) and is silent on their internals, so this file writes
out the textbook scheme step by step:

  * ring Z_Q[X]/(X^n+1) in residue form, ciphertext (c0, c1) with c0 + c1*s = m + e;
  * slots through the canonical embedding at the roots zeta_j = exp(i*pi*5^j/n);
  * Rot(c, r)[i] = c[i + r] (left shift, Sec. 2.1) through the Galois map X -> X^(5^r)
    followed by a key switch;
  * hybrid key switching: split into digits of `alpha` primes, raise each digit to the
    extended basis with the fast (non-centred, uncorrected) base conversion, multiply by
    the evaluation key, divide by the special modulus P with the floor variant;
  * rescale by the last prime, floor variant.

Polynomials are numpy uint64 arrays [limbs][n]; ciphertext and plaintext polynomials are kept
in the evaluation (NTT) domain, natural order.  The canonical form that is compared with any
other implementation is the coefficient domain with residues in [0, q).
"""
from dataclasses import dataclass
from decimal import Decimal, getcontext
from typing import Dict, List

import numpy as np

from .native import lib, p as _p, pi as _pi
from .params import Params

# stream identifiers of the counter-based generator: purpose in the top byte
ST_SECRET, ST_EVK_A, ST_EVK_E, ST_ENC_A, ST_ENC_E, ST_NOISE = 1, 2, 3, 4, 5, 6
# Which seed keys which stream.  The seed given to keygen_rotations / encrypt is PUBLIC: the uniform
# halves (a_j of a key, c1 of a ciphertext) are its streams, and the generator's finaliser is a
# bijection, so anything derived from it alone can be recomputed by whoever holds the key or the
# ciphertext.  The error polynomials are therefore drawn from the streams of (seed XOR noise), where
# noise = key(secret key's seed, ST_NOISE) is a 64-bit value only the holder of the secret key has.
# The generator is a reproducibility device (both implementations must draw identical values), not
# a cryptographic one.
RELIN_ID = 0  # evaluation-key identifier of s^2 -> s (Galois elements are odd, never 0)


def stream_id(purpose, ident=0, digit=0, limb=0):
    return (purpose << 56) | (ident << 16) | (digit << 8) | limb


def gauss_cdt(sigma: float) -> np.ndarray:
    """Cumulative table of |X| for the discrete Gaussian of parameter sigma cut at 6 sigma:
    weights w_k = exp(-k^2 / (2 sigma^2)); P(0) = w_0/Z, P(k) = 2 w_k/Z (k >= 1);
    cdt[k] = floor(2^63 * sum_{j<=k} P(j)), k = 0..kmax-1."""
    getcontext().prec = 80
    s = Decimal(repr(sigma))
    kmax = int(6 * sigma)
    w = [(-(Decimal(k) ** 2) / (2 * s * s)).exp() * (1 if k == 0 else 2) for k in range(kmax + 1)]
    z, acc, out = sum(w), Decimal(0), []
    for k in range(kmax):
        acc += w[k]
        out.append(int((acc / z) * (1 << 63)))
    return np.array(out, dtype=np.uint64)


@dataclass
class Ct:
    c: List[np.ndarray]   # components, each [level+1][n], evaluation domain
    level: int
    scale: float


@dataclass
class Pt:
    m: np.ndarray         # [level+1][n], evaluation domain
    level: int
    scale: float


@dataclass
class Evk:
    b: np.ndarray         # [digits][L+1+K][n], evaluation domain
    a: np.ndarray


class Context:
    def __init__(self, prm: Params):
        self.prm = prm
        self.n, self.S = prm.n, prm.n // 2
        self.mod = np.array(prm.moduli, dtype=np.uint64)
        self.psi = np.array(prm.psi, dtype=np.uint64)
        logn = prm.n.bit_length() - 1
        self.brev = np.array([int(format(k, f"0{logn}b")[::-1], 2) for k in range(prm.n)], dtype=np.int64)
        self.cdt = gauss_cdt(prm.sigma)
        self.rot_count = 0      # instrumentation for the op-count pins
        self.ptmul_count = 0
        # slot j <-> exponent 5^j: position u_j = (5^j mod 2n - 1)/2 among the odd exponents
        g, pos = 1, np.empty(self.S, dtype=np.int64)
        for j in range(self.S):
            pos[j] = (g - 1) // 2
            g = g * 5 % (2 * self.n)
        self.slot_pos = pos
        k = np.arange(self.n)
        self.twist = np.exp(1j * np.pi * k / self.n)    # omega^k, omega = exp(i*pi/n)

    # ---- limb index sets -------------------------------------------------------------
    def q_idx(self, level):
        return list(range(level + 1))

    def ext_idx(self, level):
        return list(range(level + 1)) + list(range(self.prm.L + 1, self.prm.L + 1 + self.prm.K))

    # ---- ring primitives on [limbs][n] arrays ---------------------------------------
    def _mods(self, idx):
        return np.ascontiguousarray(self.mod[idx]), np.ascontiguousarray(self.psi[idx])

    def ntt(self, a, idx):
        q, psi = self._mods(idx)
        out = np.array(a, dtype=np.uint64, order="C")
        lib.orc_ntt(_p(out), len(idx), self.n, _p(q), _p(psi))
        return out

    def intt(self, a, idx):
        q, psi = self._mods(idx)
        out = np.array(a, dtype=np.uint64, order="C")
        lib.orc_intt(_p(out), len(idx), self.n, _p(q), _p(psi))
        return out

    def _bin(self, fn, a, b, idx):
        q, _ = self._mods(idx)
        a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
        out = np.empty_like(a)
        fn(_p(out), _p(a), _p(b), len(idx), self.n, _p(q))
        return out

    def add(self, a, b, idx):
        return self._bin(lib.orc_add, a, b, idx)

    def sub(self, a, b, idx):
        return self._bin(lib.orc_sub, a, b, idx)

    def mul(self, a, b, idx):
        return self._bin(lib.orc_mul, a, b, idx)

    def mac(self, acc, a, b, idx):
        q, _ = self._mods(idx)
        a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
        lib.orc_mac(_p(acc), _p(a), _p(b), len(idx), self.n, _p(q))

    def mul_scalar(self, a, scalars, idx):
        q, _ = self._mods(idx)
        a = np.ascontiguousarray(a)
        c = np.array([int(s) % int(m) for s, m in zip(scalars, q)], dtype=np.uint64)
        out = np.empty_like(a)
        lib.orc_mul_scalar(_p(out), _p(a), _p(c), len(idx), self.n, _p(q))
        return out

    def automorphism_coeff(self, a, idx, g):
        q, _ = self._mods(idx)
        a = np.ascontiguousarray(a)
        out = np.empty_like(a)
        lib.orc_automorphism(_p(out), _p(a), len(idx), self.n, _p(q), g)
        return out

    def automorphism(self, a, idx, g):
        """Galois map on an evaluation-domain polynomial, by its definition on coefficients."""
        return self.ntt(self.automorphism_coeff(self.intt(a, idx), idx, g), idx)

    def from_i64(self, coeffs, idx):
        q, _ = self._mods(idx)
        c = np.ascontiguousarray(coeffs, dtype=np.int64)
        out = np.empty((len(idx), self.n), dtype=np.uint64)
        lib.orc_reduce_i64(_p(out), _pi(c), len(idx), self.n, _p(q))
        return out

    def base_conv(self, a, src, dst):
        """Fast base conversion of coefficient-domain limbs from moduli `src` to `dst`."""
        qs, qt = [int(self.mod[i]) for i in src], [int(self.mod[i]) for i in dst]
        B = 1
        for m in qs:
            B *= m
        hat = [B // m for m in qs]
        inv_hat = np.array([pow(h % m, -1, m) for h, m in zip(hat, qs)], dtype=np.uint64)
        hat_mod = np.array([[h % r for r in qt] for h in hat], dtype=np.uint64)
        a = np.ascontiguousarray(a)
        out = np.empty((len(dst), self.n), dtype=np.uint64)
        lib.orc_base_conv(_p(out), _p(a), len(src), len(dst), self.n,
                          _p(np.array(qs, dtype=np.uint64)), _p(np.array(qt, dtype=np.uint64)),
                          _p(inv_hat), _p(np.ascontiguousarray(hat_mod)))
        return out

    # ---- encoding (canonical embedding) ---------------------------------------------
    def galois(self, r):
        """Galois element of a left rotation by r slots (negative r = right rotation)."""
        return pow(5, r % self.S, 2 * self.n)

    def embed_inverse(self, z):
        """Real coefficient vector m (floats, unscaled) with m(zeta_j) = z_j."""
        v = np.zeros(self.n, dtype=np.complex128)
        zz = np.zeros(self.S, dtype=np.complex128)
        zz[:len(z)] = z
        v[self.slot_pos] = zz
        v[self.n - 1 - self.slot_pos] = np.conj(zz)     # exponent -(2u+1) = 2(n-1-u)+1 mod 2n
        return (np.fft.fft(v) * np.conj(self.twist) / self.n).real

    def encode_coeffs(self, z, scale):
        """Integer coefficients round(scale * m_k)."""
        return np.rint(self.embed_inverse(z) * scale).astype(np.int64)

    def encode(self, z, level, scale=None) -> Pt:
        scale = self.prm.scale if scale is None else scale
        return self.pt_from_coeffs(self.encode_coeffs(z, scale), level, scale)

    def pt_from_coeffs(self, coeffs, level, scale) -> Pt:
        idx = self.q_idx(level)
        return Pt(self.ntt(self.from_i64(coeffs, idx), idx), level, scale)

    def decode_coeffs(self, m_float):
        """Slot values of a real coefficient vector: z_j = sum_k m_k zeta_j^k."""
        vals = np.fft.ifft(m_float * self.twist) * self.n
        return vals[self.slot_pos]

    def centred_coeffs(self, a_coeff, level):
        """Centred integer lift (as Python ints) from the lowest one or two limbs."""
        q0 = int(self.mod[0])
        if level == 0:
            return [int(x) - q0 if int(x) > q0 // 2 else int(x) for x in a_coeff[0]]
        q1 = int(self.mod[1])
        Q, inv = q0 * q1, pow(q0, -1, q1)
        out = []
        for x0, x1 in zip(a_coeff[0].tolist(), a_coeff[1].tolist()):
            v = x0 + q0 * (((x1 - x0) * inv) % q1)
            out.append(v - Q if v > Q // 2 else v)
        return out

    # ---- keys -----------------------------------------------------------------------
    def sample_secret(self, seed) -> np.ndarray:
        """Ternary secret coefficients in {-1,0,1} (int64[n])."""
        n, h = self.n, self.prm.hamming
        st = stream_id(ST_SECRET)
        s = np.zeros(n, dtype=np.int64)
        if h == 0:
            for i in range(n):      # uniform on {0, 1, -1}: reject only the draw 2^64 - 1
                att = 0
                while True:
                    v = lib.orc_rng_draw(seed, st, (att << 32) | i)
                    if v < 3 * ((1 << 64) // 3):
                        break
                    att += 1
                s[i] = (0, 1, -1)[v % 3]
        else:                       # partial Fisher-Yates picks h positions; a draw bit the sign
            perm = list(range(n))
            for i in range(h):
                j = i + lib.orc_rng_draw(seed, st, i) % (n - i)
                perm[i], perm[j] = perm[j], perm[i]
                s[perm[i]] = -1 if lib.orc_rng_draw(seed, st, n + i) & 1 else 1
        return s

    def keygen_secret(self, seed):
        s = self.sample_secret(seed)
        all_idx = list(range(len(self.mod)))
        return {"coeffs": s, "ntt": self.ntt(self.from_i64(s, all_idx), all_idx),
                "noise": lib.orc_rng_key(seed, stream_id(ST_NOISE))}

    def _uniform(self, idx, seed, purpose, ident=0, digit=0):
        out = np.empty((len(idx), self.n), dtype=np.uint64)
        for r, i in enumerate(idx):
            lib.orc_sample_uniform(_p(out[r]), self.n, int(self.mod[i]), seed,
                                   stream_id(purpose, ident, digit, i))
        return out

    def _gauss(self, seed, purpose, ident=0, digit=0):
        e = np.empty(self.n, dtype=np.int64)
        lib.orc_sample_gauss(_pi(e), self.n, _p(self.cdt), len(self.cdt), seed,
                             stream_id(purpose, ident, digit, 0))
        return e

    def keygen_switch(self, sk, s_from_ntt, ident, seed) -> Evk:
        """Evaluation key from the secret `s_from` to sk, one pair per digit of the full chain:
        b_j = -a_j s + e_j + [P mod q_i] s_from on the limbs q_i of digit j, nothing added on
        the other limbs (P * (Q/Q_j) * ((Q/Q_j)^-1 mod Q_j) is 1 there... times P, and 0
        elsewhere).  The uniform half a_j is drawn directly in the evaluation domain: its value at
        psi^(2k+1) is draw brev(k) of its stream (the draws fill the bit-reversed order in which an
        in-place transform leaves its output).  The transform is a bijection, so this is the same
        distribution as drawing coefficients, and an implementation may then regenerate a_j from the
        seed wherever it is used instead of storing it.  The errors e_j come from the streams of
        seed XOR sk["noise"], which the public seed does not determine."""
        prm, all_idx = self.prm, list(range(len(self.mod)))
        P = 1
        for m in prm.p:
            P *= m
        digits = prm.digits(prm.L)
        bs, as_ = [], []
        for j, D in enumerate(digits):
            a = self._uniform(all_idx, seed, ST_EVK_A, ident, j)[:, self.brev]
            e = self.ntt(self.from_i64(self._gauss(seed ^ sk["noise"], ST_EVK_E, ident, j), all_idx), all_idx)
            b = self.sub(e, self.mul(a, sk["ntt"], all_idx), all_idx)
            fac = [P % int(self.mod[i]) if i in D else 0 for i in all_idx]
            b = self.add(b, self.mul_scalar(s_from_ntt, fac, all_idx), all_idx)
            bs.append(b)
            as_.append(a)
        return Evk(np.stack(bs), np.stack(as_))

    def keygen_rotations(self, sk, steps, seed, with_relin=False) -> Dict[int, Evk]:
        """Keys indexed by Galois element (and RELIN_ID for s^2 -> s)."""
        all_idx = list(range(len(self.mod)))
        keys = {}
        for r in steps:
            g = self.galois(r)
            if g not in keys:
                keys[g] = self.keygen_switch(sk, self.automorphism(sk["ntt"], all_idx, g), g, seed)
        if with_relin:
            keys[RELIN_ID] = self.keygen_switch(sk, self.mul(sk["ntt"], sk["ntt"], all_idx),
                                                RELIN_ID, seed)
        return keys

    # ---- encrypt / decrypt -----------------------------------------------------------
    def encrypt(self, sk, pt: Pt, seed) -> Ct:
        """Symmetric encryption (c0, c1) = (-a s + e + m, a); a from the streams of the (public)
        seed, e from those of seed XOR sk["noise"]."""
        idx = self.q_idx(pt.level)
        a = self.ntt(self._uniform(idx, seed, ST_ENC_A), idx)
        e = self.ntt(self.from_i64(self._gauss(seed ^ sk["noise"], ST_ENC_E), idx), idx)
        c0 = self.add(self.sub(e, self.mul(a, sk["ntt"][idx], idx), idx), pt.m, idx)
        return Ct([c0, a], pt.level, pt.scale)

    def decrypt_coeffs(self, sk, ct: Ct):
        """Centred integer coefficients of c0 + c1 s (+ c2 s^2), from the two lowest limbs."""
        lv = min(ct.level, 1)
        idx = self.q_idx(lv)
        s = sk["ntt"][idx]
        acc, spow = ct.c[0][idx].copy(), s
        for comp in ct.c[1:]:
            acc = self.add(acc, self.mul(comp[idx], spow, idx), idx)
            spow = self.mul(spow, s, idx)
        return self.centred_coeffs(self.intt(acc, idx), lv)

    def decrypt(self, sk, ct: Ct, nslots=None):
        m = np.array([float(v) for v in self.decrypt_coeffs(sk, ct)])
        z = self.decode_coeffs(m / ct.scale)
        return z if nslots is None else z[:nslots]

    def canonical(self, ct: Ct) -> np.ndarray:
        """Interchange form [component][limb][coefficient], coefficient domain."""
        idx = self.q_idx(ct.level)
        return np.stack([self.intt(c, idx) for c in ct.c])

    # ---- homomorphic operations ------------------------------------------------------
    def ct_add(self, x: Ct, y: Ct) -> Ct:
        assert x.level == y.level and len(x.c) == len(y.c)
        assert abs(x.scale / y.scale - 1) < 1e-9
        idx = self.q_idx(x.level)
        return Ct([self.add(a, b, idx) for a, b in zip(x.c, y.c)], x.level, x.scale)

    def level_drop(self, x: Ct, level) -> Ct:
        assert level <= x.level
        return Ct([c[:level + 1].copy() for c in x.c], level, x.scale)

    def mul_pt(self, x: Ct, pt: Pt) -> Ct:
        assert x.level == pt.level
        idx = self.q_idx(x.level)
        self.ptmul_count += 1
        return Ct([self.mul(c, pt.m, idx) for c in x.c], x.level, x.scale * pt.scale)

    def mac_pt(self, acc: Ct, x: Ct, pt: Pt):
        """acc += x * pt (acc already at the product scale)."""
        idx = self.q_idx(x.level)
        self.ptmul_count += 1
        for a, c in zip(acc.c, x.c):
            self.mac(a, c, pt.m, idx)

    def mul_ct(self, x: Ct, y: Ct) -> Ct:
        """Tensor product (c0 d0, c0 d1 + c1 d0, c1 d1), not yet relinearised."""
        assert x.level == y.level and len(x.c) == 2 and len(y.c) == 2
        idx = self.q_idx(x.level)
        d0 = self.mul(x.c[0], y.c[0], idx)
        d1 = self.add(self.mul(x.c[0], y.c[1], idx), self.mul(x.c[1], y.c[0], idx), idx)
        d2 = self.mul(x.c[1], y.c[1], idx)
        return Ct([d0, d1, d2], x.level, x.scale * y.scale)

    def rescale(self, x: Ct) -> Ct:
        """Divide by the last prime q_l, floor variant:
        c'_i = (c_i - [c_l]_{q_i}) * q_l^{-1} mod q_i, with c_l lifted to [0, q_l)."""
        l = x.level
        assert l >= 1
        idx, ql = self.q_idx(l - 1), int(self.mod[l])
        inv = [pow(ql, -1, int(self.mod[i])) for i in idx]
        out = []
        for c in x.c:
            last = self.intt(c[l:l + 1], [l])
            q, _ = self._mods(idx)
            red = np.empty((len(idx), self.n), dtype=np.uint64)
            lib.orc_reduce_u64(_p(red), _p(last), len(idx), self.n, _p(q))
            diff = self.sub(c[:l], self.ntt(red, idx), idx)
            out.append(self.mul_scalar(diff, inv, idx))
        return Ct(out, l - 1, x.scale / ql)

    # ---- hybrid key switching --------------------------------------------------------
    def modup(self, d_coeff, level):
        """Raise each digit of a coefficient-domain polynomial [level+1][n] to the extended
        basis (q_0..q_level, p_0..p_{K-1}); own limbs are copied.  Returns coefficient-domain
        arrays [digits][level+1+K][n]."""
        ext = self.ext_idx(level)
        out = []
        for D in self.prm.digits(level):
            others = [i for i in ext if i not in D]
            conv = self.base_conv(d_coeff[D], D, others)
            full = np.empty((len(ext), self.n), dtype=np.uint64)
            for r, i in enumerate(ext):
                full[r] = d_coeff[i] if i in D else conv[others.index(i)]
            out.append(full)
        return out

    def moddown(self, u, level):
        """(u - Conv_{P->Q}([u]_P)) * P^{-1} on an evaluation-domain [level+1+K][n] array."""
        prm = self.prm
        qi, sp = self.q_idx(level), list(range(prm.L + 1, prm.L + 1 + prm.K))
        conv = self.base_conv(self.intt(u[level + 1:], sp), sp, qi)
        P = 1
        for m in prm.p:
            P *= m
        inv = [pow(P % int(self.mod[i]), -1, int(self.mod[i])) for i in qi]
        return self.mul_scalar(self.sub(u[:level + 1], self.ntt(conv, qi), qi), inv, qi)

    def inner_product(self, digits_ntt, evk: Evk, level):
        ext = self.ext_idx(level)
        u0 = np.zeros((len(ext), self.n), dtype=np.uint64)
        u1 = np.zeros_like(u0)
        for j, d in enumerate(digits_ntt):
            self.mac(u0, d, evk.b[j][ext], ext)
            self.mac(u1, d, evk.a[j][ext], ext)
        return u0, u1

    def keyswitch(self, d, level, evk: Evk):
        """(ks0, ks1) with ks0 + ks1 s = d * s_from + small, for evaluation-domain d."""
        ext = self.ext_idx(level)
        digits = [self.ntt(x, ext) for x in self.modup(self.intt(d, self.q_idx(level)), level)]
        u0, u1 = self.inner_product(digits, evk, level)
        return self.moddown(u0, level), self.moddown(u1, level)

    def relinearize(self, x: Ct, keys) -> Ct:
        assert len(x.c) == 3
        idx = self.q_idx(x.level)
        k0, k1 = self.keyswitch(x.c[2], x.level, keys[RELIN_ID])
        return Ct([self.add(x.c[0], k0, idx), self.add(x.c[1], k1, idx)], x.level, x.scale)

    def rotate(self, x: Ct, r, keys) -> Ct:
        """Rot(x, r): Galois map on both components, then key switch of the second one."""
        assert len(x.c) == 2
        g, idx = self.galois(r), self.q_idx(x.level)
        self.rot_count += 1
        c0 = self.automorphism(x.c[0], idx, g)
        c1 = self.automorphism(x.c[1], idx, g)
        k0, k1 = self.keyswitch(c1, x.level, keys[g])
        return Ct([self.add(c0, k0, idx), k1], x.level, x.scale)

    def hoist(self, x: Ct):
        """Shared part of several rotations of one ciphertext: the raised digits of c1
        (coefficient domain).  The Galois map is then applied to the raised digits, which is
        NOT bit-identical to raising the mapped polynomial (the fast conversion of -a is not
        minus the conversion of a), though both decrypt to the same rotation."""
        return self.modup(self.intt(x.c[1], self.q_idx(x.level)), x.level)

    def rotate_hoisted(self, x: Ct, hoisted, r, keys) -> Ct:
        g, idx, ext = self.galois(r), self.q_idx(x.level), self.ext_idx(x.level)
        self.rot_count += 1
        digits = [self.ntt(self.automorphism_coeff(d, ext, g), ext) for d in hoisted]
        u0, u1 = self.inner_product(digits, keys[g], x.level)
        c0 = self.automorphism(x.c[0], idx, g)
        return Ct([self.add(c0, self.moddown(u0, x.level), idx), self.moddown(u1, x.level)],
                  x.level, x.scale)

    # ---- accumulation in the raised basis (double hoisting) -----------------------------------
    # App. C notes that more than half of the rotations of the packed product act on one
    # ciphertext and can share their ModUp; the paper does not say where their ModDown goes.
    # The reading taken here postpones it: a hoisted rotation is left in the extended basis
    # (q_0..q_level, p_0..p_{K-1}) as
    #       R = (u0 + P * sigma(c0),  u1),        ModDown(R) = rotate_hoisted(x) exactly,
    # the plaintext products are summed there, and the division by P happens once per giant
    # step, inside that step's own key switch (ModDown is additive up to rounding).
    def _P(self):
        P = 1
        for m in self.prm.p:
            P *= m
        return P

    def pt_from_coeffs_ext(self, coeffs, level, scale) -> Pt:
        """The plaintext polynomial on all limbs of the extended basis at `level`."""
        ext = self.ext_idx(level)
        return Pt(self.ntt(self.from_i64(coeffs, ext), ext), level, scale)

    def encode_ext(self, z, level, scale=None) -> Pt:
        scale = self.prm.scale if scale is None else scale
        return self.pt_from_coeffs_ext(self.encode_coeffs(z, scale), level, scale)

    def raise_ct(self, x: Ct):
        """(P c0, P c1) in the extended basis: residues P*c mod q_i, zero on the special limbs."""
        assert len(x.c) == 2
        ext, nq = self.ext_idx(x.level), x.level + 1
        P = self._P()
        out = []
        for c in x.c:
            full = np.zeros((len(ext), self.n), dtype=np.uint64)
            full[:nq] = self.mul_scalar(c, [P] * nq, self.q_idx(x.level))
            out.append(full)
        return out

    def rotate_hoisted_raised(self, x: Ct, hoisted, r, keys):
        """The hoisted rotation by r before its ModDown: [u0 + P sigma(c0), u1], each [ext][n]."""
        g, idx, ext = self.galois(r), self.q_idx(x.level), self.ext_idx(x.level)
        self.rot_count += 1
        digits = [self.ntt(self.automorphism_coeff(d, ext, g), ext) for d in hoisted]
        u0, u1 = self.inner_product(digits, keys[g], x.level)
        nq = x.level + 1
        u0[:nq] = self.add(u0[:nq], self.mul_scalar(self.automorphism(x.c[0], idx, g), [self._P()] * nq, idx), idx)
        return [u0, u1]

    def hoist_raised(self, R, level):
        """Shared part of several rotations of a ciphertext held in the extended basis (R ~ P ct):
        the second component alone is divided by P, and its digits are raised."""
        return self.modup(self.intt(self.moddown(R[1], level), self.q_idx(level)), level)

    def rotate_raised_hoisted(self, R, hoisted, level, r, keys):
        """Rotation of a ciphertext that is held in the extended basis and stays there: the first
        component goes through the Galois map on all limbs and joins the key-switch sum as it is,
              [u0 + sigma(R0), u1],   u = sum_d sigma(digits_d(ModDown(R1))) * key_d.
        P * ModDown(R0) and R0 differ by the lift of R0 mod P, less than K P, so after the ModDown
        that ends the sum the result is Rot(ModDown(R), r) up to a few units of rounding in the
        first component (and exactly that when R0 vanishes on the special limbs)."""
        g, ext = self.galois(r), self.ext_idx(level)
        self.rot_count += 1
        digits = [self.ntt(self.automorphism_coeff(d, ext, g), ext) for d in hoisted]
        u0, u1 = self.inner_product(digits, keys[g], level)
        return [self.add(u0, self.automorphism(R[0], ext, g), ext), u1]

    def rotate_raised(self, R, level, r, keys):
        return self.rotate_raised_hoisted(R, self.hoist_raised(R, level), level, r, keys)

    def rotsum_raised(self, R, level, amounts, keys):
        """R + sum_a Rot(R, a) in the extended basis, all rotations sharing one set of raised digits."""
        ext = self.ext_idx(level)
        hoisted = self.hoist_raised(R, level)
        acc = [R[0].copy(), R[1].copy()]
        for a in amounts:
            T = self.rotate_raised_hoisted(R, hoisted, level, a, keys)
            acc = [self.add(acc[0], T[0], ext), self.add(acc[1], T[1], ext)]
        return acc

    def mac_pt_raised(self, acc, R, pt: Pt, level):
        """acc += R * pt on the extended basis (acc, R: two [ext][n] arrays; pt from *_ext)."""
        ext = self.ext_idx(level)
        self.ptmul_count += 1
        for a, c in zip(acc, R):
            self.mac(a, c, pt.m, ext)

    def moddown_ct(self, R, level, scale) -> Ct:
        return Ct([self.moddown(R[0], level), self.moddown(R[1], level)], level, scale)

    def rotate_add_raised(self, x: Ct, r, keys, E) -> Ct:
        """Rot(x, r) + ModDown(E) with one ModDown: E (two [ext][n] arrays) joins the key-switch
        sum before the division by P."""
        assert len(x.c) == 2
        g, idx, ext = self.galois(r), self.q_idx(x.level), self.ext_idx(x.level)
        self.rot_count += 1
        c0 = self.automorphism(x.c[0], idx, g)
        c1 = self.automorphism(x.c[1], idx, g)
        digits = [self.ntt(d, ext) for d in self.modup(self.intt(c1, idx), x.level)]
        u0, u1 = self.inner_product(digits, keys[g], x.level)
        u0, u1 = self.add(u0, E[0], ext), self.add(u1, E[1], ext)
        return Ct([self.add(c0, self.moddown(u0, x.level), idx), self.moddown(u1, x.level)], x.level, x.scale)
