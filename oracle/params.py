"""Oracle: RNS-CKKS parameter sets (TEST INFRASTRUCTURE).

The paper fixes only the ring degree, the slot count and the bit sizes of the modulus
chain (Sec. 7.1, "Cryptographic Configuration"); the workloads' own chains are stated by
the benchmark configurations.  Primes are chosen by a deterministic rule so that two
independent implementations arrive at the same chain:

    candidates 2^bits + 1 - k*2n for k = 1, 2, 3, ...; keep the primes, in that order.

All of them satisfy q = 1 (mod 2n), so X^n + 1 splits completely.
"""
from dataclasses import dataclass, field
from typing import List


def is_prime(m: int) -> bool:
    """Deterministic Miller-Rabin for m < 2^64 (first twelve prime bases)."""
    if m < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)
    for s in small:
        if m % s == 0:
            return m == s
    d, r = m - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in small:
        x = pow(a, d, m)
        if x in (1, m - 1):
            continue
        for _ in range(r - 1):
            x = x * x % m
            if x == m - 1:
                break
        else:
            return False
    return True


def scan_primes(bits: int, n: int, count: int) -> List[int]:
    out, k = [], 1
    while len(out) < count:
        c = (1 << bits) + 1 - k * 2 * n
        if is_prime(c):
            out.append(c)
        k += 1
    return out


def primitive_2n_root(q: int, n: int) -> int:
    """Smallest-base psi = x^((q-1)/2n) with psi^n = -1 (so psi has order exactly 2n)."""
    x = 2
    while True:
        psi = pow(x, (q - 1) // (2 * n), q)
        if pow(psi, n, q) == q - 1:
            return psi
        x += 1


@dataclass
class Params:
    n: int                      # ring degree (the paper's N')
    q: List[int]                # ciphertext primes q_0..q_L
    p: List[int]                # special primes p_0..p_{K-1}
    alpha: int                  # primes per key-switch digit
    scale: float                # default encoding scale (Delta)
    hamming: int = 0            # 0: i.i.d. uniform ternary secret; h>0: exactly h non-zeros
    sigma: float = 3.2
    name: str = ""
    psi: List[int] = field(default_factory=list)   # 2n-th roots for q + p

    def __post_init__(self):
        assert self.n & (self.n - 1) == 0
        for m in self.q + self.p:
            assert (m - 1) % (2 * self.n) == 0 and is_prime(m)
        assert len(set(self.q + self.p)) == len(self.q) + len(self.p)
        if not self.psi:
            self.psi = [primitive_2n_root(m, self.n) for m in self.q + self.p]

    @property
    def slots(self):
        return self.n // 2

    @property
    def L(self):
        return len(self.q) - 1

    @property
    def K(self):
        return len(self.p)

    @property
    def moduli(self):
        return self.q + self.p

    def digits(self, level: int):
        """Key-switch digits at a level: lists of limb indices, alpha per digit."""
        return [list(range(s, min(s + self.alpha, level + 1)))
                for s in range(0, level + 1, self.alpha)]


def toy(n=4096, q0_bits=50, qi_bits=40, n_qi=4, p_bits=60, n_p=1, alpha=1, scale_bits=40,
        hamming=0, name="toy"):
    """Small ring in the shape of benchmark configuration 1: a q0_bits base prime, n_qi
    primes of qi_bits, n_p special primes.  With a single special prime the digits hold one
    prime each (alpha = 1): a single digit covering the whole 210-bit chain against one
    60-bit special prime leaves key-switch noise far above the scale."""
    q = scan_primes(q0_bits, n, 1) + scan_primes(qi_bits, n, n_qi)
    return Params(n=n, q=q, p=scan_primes(p_bits, n, n_p), alpha=alpha,
                  scale=float(2 ** scale_bits), hamming=hamming, name=name)


def config1():
    return toy(name="config1")


def llama_ring(n_q=24, n_p=4, n=65536, name="config2"):
    """Benchmark configurations 2-4 (24 + 4 primes) and 5 (36 + 6): 50-bit ciphertext primes,
    60-bit special primes, dnum = 6 digits, scale 2^50, secret of Hamming weight 192."""
    assert n_q % 6 == 0
    return Params(n=n, q=scan_primes(50, n, n_q), p=scan_primes(60, n, n_p), alpha=n_q // 6,
                  scale=float(2 ** 50), hamming=192, name=name)


def config2():
    return llama_ring(24, 4, name="config2")


def config5():
    return llama_ring(36, 6, name="config5")
