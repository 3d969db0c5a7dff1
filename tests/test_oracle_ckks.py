"""Pins for the oracle's CKKS scheme: direct definitions, big-int CRT and decrypted meaning."""
import math
import random

import numpy as np
import pytest

from oracle import ckks, params


@pytest.fixture(scope="module")
def small():
    prm = params.toy(n=64, n_qi=5, n_p=2, alpha=2, scale_bits=30)
    ctx = ckks.Context(prm)
    return ctx, ctx.keygen_secret(3)


@pytest.fixture(scope="module")
def mid():
    prm = params.config1()
    ctx = ckks.Context(prm)
    sk = ctx.keygen_secret(7)
    keys = ctx.keygen_rotations(sk, [1, -1, 7, ctx.S // 2, ctx.S - 1], 5, with_relin=True)
    return ctx, sk, keys


def big(ctx, a_coeff, idx):
    """CRT lift of coefficient-domain residues to integers in [0, prod q)."""
    qs = [int(ctx.mod[i]) for i in idx]
    Q = math.prod(qs)
    out = []
    for c in range(a_coeff.shape[1]):
        v = sum(int(a_coeff[r, c]) * (Q // q) * pow(Q // q, -1, q) for r, q in enumerate(qs)) % Q
        out.append(v)
    return out, Q


@pytest.mark.parametrize("n", [8, 64])
def test_encode_against_direct_embedding_definition(n):
    ctx = ckks.Context(params.toy(n=n))
    S = n // 2
    rng = np.random.default_rng(n)
    z = rng.normal(size=S) + 1j * rng.normal(size=S)
    omega = np.exp(1j * np.pi / n)
    zeta = np.array([omega ** pow(5, j, 2 * n) for j in range(S)])
    m_direct = np.array([(z * np.conj(zeta ** k)).sum().real / S for k in range(n)])
    assert np.allclose(ctx.embed_inverse(z), m_direct, atol=1e-12)
    # decode definition z_j = m(zeta_j)
    dec = np.array([(m_direct * zeta[j] ** np.arange(n)).sum() for j in range(S)])
    assert np.allclose(dec, z, atol=1e-12)
    assert np.allclose(ctx.decode_coeffs(m_direct), z, atol=1e-12)
    coeffs = ctx.encode_coeffs(z, 2.0 ** 30)
    assert np.abs(coeffs - m_direct * 2.0 ** 30).max() <= 0.5 + 1e-3


def test_encode_decode_roundtrip_large():
    ctx = ckks.Context(params.config1())
    rng = np.random.default_rng(0)
    z = rng.uniform(-1, 1, ctx.S)
    m = ctx.encode_coeffs(z, 2.0 ** 40).astype(np.float64)
    assert np.abs(ctx.decode_coeffs(m / 2.0 ** 40) - z).max() < 2.0 ** -28


def test_slot_product_is_ring_product(small):
    ctx, _ = small
    rng = np.random.default_rng(1)
    z1, z2 = rng.normal(size=ctx.S), rng.normal(size=ctx.S)
    idx = ctx.q_idx(2)
    a, b = ctx.encode(z1, 2), ctx.encode(z2, 2)
    prod = ctx.intt(ctx.mul(a.m, b.m, idx), idx)
    m = np.array([float(v) for v in ctx.centred_coeffs(prod, 1)])
    assert np.abs(ctx.decode_coeffs(m / (a.scale * b.scale)) - z1 * z2).max() < 1e-6


def test_decrypt_of_encrypt_and_noise_size(mid):
    ctx, sk, _ = mid
    rng = np.random.default_rng(2)
    z = rng.uniform(-1, 1, ctx.S)
    pt = ctx.encode(z, ctx.prm.L)
    ct = ctx.encrypt(sk, pt, 11)
    assert np.abs(ctx.decrypt(sk, ct) - z).max() < 1e-8
    noise = np.array(ctx.decrypt_coeffs(sk, ct), dtype=np.float64) - ctx.encode_coeffs(z, pt.scale)
    assert abs(noise.std() - ctx.prm.sigma) < 0.2        # c0 + c1 s - m = e exactly
    assert np.abs(noise).max() <= 19
    assert np.array_equal(noise.astype(np.int64), ctx._gauss(11 ^ sk["noise"], ckks.ST_ENC_E))
    # c1 is the uniform sample itself, in the coefficient domain
    can = ctx.canonical(ct)
    assert np.array_equal(can[1], ctx._uniform(ctx.q_idx(ctx.prm.L), 11, ckks.ST_ENC_A))
    # fresh randomness per seed
    assert not np.array_equal(ctx.canonical(ctx.encrypt(sk, pt, 12))[1], can[1])


def test_modup_residues_are_lift_plus_small_multiple_of_digit_modulus(small):
    ctx, _ = small
    prm = ctx.prm
    rng = random.Random(4)
    for level in (prm.L, 2):
        idx, ext = ctx.q_idx(level), ctx.ext_idx(level)
        d = np.array([[rng.randrange(int(ctx.mod[i])) for _ in range(ctx.n)] for i in idx],
                     dtype=np.uint64)
        raised = ctx.modup(d, level)
        digits = prm.digits(level)
        assert len(raised) == len(digits) and sum(len(D) for D in digits) == level + 1
        for D, full in zip(digits, raised):
            vals, QD = big(ctx, d[D], D)
            for c in range(ctx.n):
                es = {(int(full[r, c]) - vals[c]) * pow(QD, -1, int(ctx.mod[i])) % int(ctx.mod[i])
                      for r, i in enumerate(ext) if i not in D}
                assert len(es) == 1 and es.pop() < len(D)
            for r, i in enumerate(ext):
                if i in D:
                    assert np.array_equal(full[r], d[i])


def test_moddown_divides_by_P_with_floor(small):
    ctx, _ = small
    prm = ctx.prm
    P = math.prod(prm.p)
    level = 3
    ext, idx = ctx.ext_idx(level), ctx.q_idx(level)
    rng = random.Random(6)
    QP = math.prod(int(ctx.mod[i]) for i in ext)
    vals = [rng.randrange(QP) for _ in range(ctx.n)]
    vals[0], vals[1], vals[2] = 0, P * 12345, P * 777 + P - 1
    u = np.array([[v % int(ctx.mod[i]) for v in vals] for i in ext], dtype=np.uint64)
    out = ctx.intt(ctx.moddown(ctx.ntt(u, ext), level), idx)
    for c, v in enumerate(vals):
        # floor(v / P) up to the fast conversion's overshoot: (v - ([v]_P + e P)) / P, 0 <= e < K
        cands = [[((v // P) - e) % int(ctx.mod[i]) for i in idx] for e in range(prm.K)]
        assert out[:, c].tolist() in cands
    assert out[:, 0].tolist() == [0] * len(idx)
    assert out[:, 1].tolist() == [12345 % int(ctx.mod[i]) for i in idx]


def test_rescale_is_floor_division_by_last_prime(small):
    ctx, sk = small
    level = 3
    idx = ctx.q_idx(level)
    rng = random.Random(7)
    Q = math.prod(int(ctx.mod[i]) for i in idx)
    vals = [rng.randrange(Q) for _ in range(ctx.n)]
    a = np.array([[v % int(ctx.mod[i]) for v in vals] for i in idx], dtype=np.uint64)
    ct = ckks.Ct([ctx.ntt(a, idx), ctx.ntt(a, idx)], level, 2.0 ** 60)
    out = ctx.rescale(ct)
    ql = int(ctx.mod[level])
    assert out.level == level - 1 and out.scale == 2.0 ** 60 / ql
    got = ctx.intt(out.c[0], ctx.q_idx(level - 1))
    for c, v in enumerate(vals):
        assert got[:, c].tolist() == [(v // ql) % int(ctx.mod[i]) for i in range(level)]


def test_evaluation_key_structure(small):
    """b_j + a_j s = e_j + P * s_from on the limbs of digit j, e_j alone elsewhere."""
    ctx, sk = small
    prm = ctx.prm
    all_idx = list(range(len(ctx.mod)))
    g = ctx.galois(3)
    evk = ctx.keygen_rotations(sk, [3], 9)[g]
    s_from = ctx.automorphism_coeff(ctx.from_i64(sk["coeffs"], all_idx), all_idx, g)
    P = math.prod(prm.p)
    digits = prm.digits(prm.L)
    assert evk.b.shape == (len(digits), len(all_idx), ctx.n)
    for j, D in enumerate(digits):
        lhs = ctx.intt(ctx.add(evk.b[j], ctx.mul(evk.a[j], sk["ntt"], all_idx), all_idx), all_idx)
        e = ctx._gauss(9 ^ sk["noise"], ckks.ST_EVK_E, g, j)      # the errors: streams of seed XOR the secret key's value
        for i in all_idx:
            q = int(ctx.mod[i])
            want = [(int(e[c]) + (P * int(s_from[i, c]) if i in D else 0)) % q
                    for c in range(ctx.n)]
            assert lhs[i].tolist() == want
    # the uniform half is the generator's stream itself: the value at psi^(2k+1) is draw brev(k)
    # (what lets an implementation regenerate it from the seed instead of storing it)
    logn = ctx.n.bit_length() - 1
    brev = [int(format(k, f"0{logn}b")[::-1], 2) for k in range(ctx.n)]
    for j in range(len(digits)):
        u = ctx._uniform(all_idx, 9, ckks.ST_EVK_A, g, j)
        assert all(np.array_equal(evk.a[j][:, k], u[:, brev[k]]) for k in (0, 1, 2, 5, ctx.n - 1))
        assert np.array_equal(evk.a[j][:, brev], u)


@pytest.mark.parametrize("level", [4, 2, 0])
def test_keyswitch_changes_the_key_not_the_message(mid, level):
    ctx, sk, keys = mid
    idx = ctx.q_idx(level)
    rng = np.random.default_rng(level)
    d = (rng.integers(0, 1 << 62, (level + 1, ctx.n), dtype=np.uint64) % ctx.mod[idx][:, None])
    d = d.astype(np.uint64)
    g = ctx.galois(7)
    s_from = ctx.automorphism(sk["ntt"], list(range(len(ctx.mod))), g)[idx]
    k0, k1 = ctx.keyswitch(d, level, keys[g])
    lhs = ctx.add(k0, ctx.mul(k1, sk["ntt"][idx], idx), idx)
    diff = ctx.intt(ctx.sub(lhs, ctx.mul(d, s_from, idx), idx), idx)
    centred = np.array(ctx.centred_coeffs(diff, min(level, 1)), dtype=np.float64)
    # noise: digits * n * q_digit * sigma / P  plus the rounding term (1 + |s|_1)/2
    assert np.abs(centred).max() < 2 ** 20


@pytest.mark.parametrize("r", [1, -1, 7, 1024, 2047])
def test_rotation_is_cyclic_left_shift_of_slots(mid, r):
    ctx, sk, keys = mid
    rng = np.random.default_rng(3)
    z = rng.uniform(-1, 1, ctx.S) + 1j * rng.uniform(-1, 1, ctx.S)
    ct = ctx.encrypt(sk, ctx.encode(z, ctx.prm.L), 21)
    out = ctx.decrypt(sk, ctx.rotate(ct, r, keys))
    want = np.array([z[(i + r) % ctx.S] for i in range(ctx.S)])     # Rot(c, r)[i] = c[i + r]
    assert np.abs(out - want).max() < 1e-6
    assert np.abs(out - z).max() > 0.1


def test_hoisted_rotation_same_message_different_limbs(mid):
    ctx, sk, keys = mid
    rng = np.random.default_rng(4)
    z = rng.uniform(-1, 1, ctx.S)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(z, ctx.prm.L), 22), 3)
    h = ctx.hoist(ct)
    a, b = ctx.rotate_hoisted(ct, h, 7, keys), ctx.rotate(ct, 7, keys)
    assert np.abs(ctx.decrypt(sk, a) - np.roll(z, -7)).max() < 1e-6
    assert np.abs(ctx.decrypt(sk, b) - np.roll(z, -7)).max() < 1e-6
    assert a.level == b.level == 3


def test_ct_ct_multiplication_relinearisation_and_rescale(mid):
    ctx, sk, keys = mid
    rng = np.random.default_rng(5)
    z1, z2 = rng.uniform(-1, 1, ctx.S), rng.uniform(-1, 1, ctx.S)
    L = ctx.prm.L
    a = ctx.encrypt(sk, ctx.encode(z1, L), 31)
    b = ctx.encrypt(sk, ctx.encode(z2, L), 32)
    t = ctx.mul_ct(a, b)
    assert np.abs(ctx.decrypt(sk, t) - z1 * z2).max() < 1e-6       # three-component decrypt
    m = ctx.rescale(ctx.relinearize(t, keys))
    assert m.level == L - 1 and len(m.c) == 2
    assert np.abs(ctx.decrypt(sk, m) - z1 * z2).max() < 1e-6
    mp = ctx.rescale(ctx.mul_pt(a, ctx.encode(z2, L)))
    assert np.abs(ctx.decrypt(sk, mp) - z1 * z2).max() < 1e-6
    s = ctx.ct_add(a, b)
    assert np.abs(ctx.decrypt(sk, s) - (z1 + z2)).max() < 1e-8


def test_single_digit_with_one_special_prime_does_not_decrypt():
    """Why configuration 1 is read as one prime per digit: a literal single digit over the
    whole chain against one special prime drowns the message."""
    prm = params.toy(n=256, alpha=5)
    ctx = ckks.Context(prm)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, [1], 2)
    z = np.random.default_rng(0).uniform(-1, 1, ctx.S)
    ct = ctx.encrypt(sk, ctx.encode(z, prm.L), 3)
    assert np.abs(ctx.decrypt(sk, ctx.rotate(ct, 1, keys)) - np.roll(z, -1)).max() > 1e6


def _unmix(z):
    """Inverse of the generator's finaliser (the SplitMix64 output function is a bijection on 64-bit words)."""
    M = (1 << 64) - 1

    def unshift(v, s):
        out = v
        for _ in range(64 // s + 1):
            out = v ^ (out >> s)
        return out
    z = unshift(z, 31)
    z = z * pow(0x94D049BB133111EB, -1, 1 << 64) & M
    z = unshift(z, 27)
    z = z * pow(0xBF58476D1CE4E5B9, -1, 1 << 64) & M
    return unshift(z, 30)


def test_the_public_seed_does_not_give_the_error_streams(small):
    """What an evaluation key or a ciphertext publishes (the uniform half, hence its stream key, hence --
    the finaliser being invertible -- the seed of the call) must not determine the error polynomials: they
    are the streams of seed XOR a value derived from the SECRET key's seed."""
    from oracle.native import lib
    ctx, sk = small
    seed, g = 0x1234, ctx.galois(3)
    # the attack the plain scheme allowed: stream key of a_0 -> mix(seed) -> seed
    stream = ckks.stream_id(ckks.ST_EVK_A, g, 0, 0)
    key = lib.orc_rng_key(seed, stream)
    assert _unmix(_unmix(key) ^ stream) == seed
    evk = ctx.keygen_rotations(sk, [3], seed)[g]
    all_idx = list(range(len(ctx.mod)))
    s_from = ctx.automorphism_coeff(ctx.from_i64(sk["coeffs"], all_idx), all_idx, g)
    P = math.prod(ctx.prm.p)
    D = ctx.prm.digits(ctx.prm.L)[0]
    lhs = ctx.intt(ctx.add(evk.b[0], ctx.mul(evk.a[0], sk["ntt"], all_idx), all_idx), all_idx)
    q0 = int(ctx.mod[0])
    e_true = [(int(lhs[0, c]) - P * int(s_from[0, c])) % q0 for c in range(ctx.n)]
    e_true = [v - q0 if v > q0 // 2 else v for v in e_true]
    assert 0 in D
    assert e_true == ctx._gauss(seed ^ sk["noise"], ckks.ST_EVK_E, g, 0).tolist()
    assert e_true != ctx._gauss(seed, ckks.ST_EVK_E, g, 0).tolist()          # the recovered seed alone is not enough
    # the value mixed in belongs to the secret key: another secret, other errors under the same public seed
    sk2 = ctx.keygen_secret(4)
    assert sk2["noise"] != sk["noise"] and sk["noise"] == lib.orc_rng_key(3, ckks.stream_id(ckks.ST_NOISE))
    ct1, ct2 = ctx.encrypt(sk, ctx.encode(np.zeros(ctx.S), 2), 77), ctx.encrypt(sk2, ctx.encode(np.zeros(ctx.S), 2), 77)
    assert np.array_equal(ct1.c[1], ct2.c[1])                                 # same public half
    n1 = np.array(ctx.decrypt_coeffs(sk, ct1)), np.array(ctx.decrypt_coeffs(sk2, ct2))
    assert not np.array_equal(n1[0], n1[1])
