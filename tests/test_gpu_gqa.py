"""GPU parity of grouped-query attention on a cache that stores every KV head once (cm_gqa_*), and of caches
whose head count is padded to a power of two: limbs against the oracle on the config-1 ring, decrypted results
against float64 on the full ring at the stated shapes of benchmark configuration 3 (32 query heads on 8 KV
heads, 128 dims, context 1024) and of GPT2-base attention (12 heads of 64 dims)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import ckks, params
    from paper_2602_11470_amd import binding as B
    prm = params.config1()
    octx, gctx = ckks.Context(prm), B.config1()
    yield dict(B=B, octx=octx, gctx=gctx, osk=octx.keygen_secret(1), gsk=gctx.keygen_secret(1), prm=prm)
    gctx.close()


def _enc_both(e, slots, level, seed):
    octx, gctx = e["octx"], e["gctx"]
    scale, top = octx.prm.scale, octx.prm.L
    coeffs = octx.encode_coeffs(slots, scale)
    o = octx.level_drop(octx.encrypt(e["osk"], octx.pt_from_coeffs(coeffs, top, scale), seed), level)
    g = gctx.encrypt(e["gsk"], gctx.pt_from_coeffs(coeffs, top, scale), seed)
    return o, (gctx.level_drop(g, level) if level != top else g)


def _same(e, o, g):
    assert g.level == o.level and abs(g.scale / o.scale - 1) < 1e-12
    assert np.array_equal(e["gctx"].ct_export(g), e["octx"].canonical(o))


@pytest.mark.parametrize("unrolled,r_i,index", [(False, 4, False), (True, 0, False), (False, 4, True), (True, 4, True)])
def test_gqa_products_match_oracle_and_float64(env, unrolled, r_i, index):
    """8 query heads on 2 KV heads of 16 dims (G = 4, t_kv = 64, t = 16) on the 2048-slot ring: the four score
    ciphertexts of q K^T and the output of scores V limb for limb against the oracle's composition of the same
    steps, and against the einsum with shared KV heads."""
    from oracle import packing, vmm
    from oracle.ckks import Pt
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    H, Hkv, E, ntok, L = 8, 2, 16, 150, octx.prm.L
    glay = packing.GqaLayout(octx.S, H, Hkv, E, r_i)
    kvl, G = glay.kv, glay.G
    rng = np.random.default_rng(61)
    q = rng.normal(size=(H, E)) * 0.3
    K, V = rng.normal(size=(ntok, Hkv, E)), rng.normal(size=(ntok, Hkv, E))
    s = rng.uniform(0, 1, size=(H, ntok))
    s /= s.sum(axis=1, keepdims=True)
    lv = L - 1
    kv = gctx.kv_create(Hkv, E, lv, r_i=r_i, unrolled_ladders=unrolled, key_index=index)
    rot_coeffs = {}
    for d_, level in ((0, lv + 1), (1, lv - 1)):
        ql = float(octx.mod[level])
        for delta in range(1, G):
            rot_coeffs[d_, delta] = [octx.encode_coeffs(p, ql) for p in kvl.inner_rotation_plaintexts(glay.inner_delta(delta))]
    gqa = gctx.gqa(kv, G, coeffs=np.stack([np.stack(rot_coeffs[d_, delta]) for d_ in (0, 1) for delta in range(1, G)]))
    steps = sorted({a for a in kv.steps() if a % kvl.t == 0} | set(gqa.steps()))
    assert set(glay.qk_steps()) | set(glay.sv_steps()) <= set(steps) or unrolled or index
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    m0 = np.zeros(octx.S)
    m0[:Hkv * kvl.t] = 1
    base = octx.encode_coeffs(m0, float(octx.mod[lv - 1]))
    kv.set_mask(0, base)

    def omask(c):
        idx = octx.q_idx(lv - 1)
        coeff = octx.automorphism_coeff(octx.from_i64(base, idx), idx, octx.galois(-(c % E) * Hkv * kvl.t))
        return Pt(octx.ntt(coeff, idx), lv - 1, float(octx.mod[lv - 1]))

    def opts(d_, level):
        ql = float(octx.mod[level])
        return {delta: [octx.pt_from_coeffs(cf, level, ql) for cf in rot_coeffs[d_, delta]] for delta in range(1, G)}
    nk = -(-ntok // kvl.t)
    okc, ovc = [], []
    for c in range(nk):
        ok, gk = _enc_both(e, kvl.pack_k(K, c), lv, 100 + c)
        okc.append(ok)
        kv.load(B.CM_QK, c, gk)
    oxc = []
    for k in range(E):
        ov, gv = _enc_both(e, kvl.pack_v(V, k), lv, 300 + k)
        ovc.append(ov)
        kv.load(B.CM_SV, k, gv)
        if index:
            ox, gx = _enc_both(e, kvl.pack_k_index(K, k), lv, 700 + k)
            oxc.append(ox)
            kv.load(B.CM_KV_INDEX, k, gx)
    kv.set_tokens(ntok)
    ops = vmm.CkksOps(octx, okeys)
    oq, gq = _enc_both(e, glay.q.pack_vec(q), lv + 1, 10)
    masks = [omask(c) for c in range(nk)]
    qk = (lambda x: vmm.qk_scores_unrolled(octx, okeys, kvl, x, okc, masks, replicate=False)) if unrolled else None
    if index and unrolled:
        qk = lambda x: vmm.score_times_v_unrolled(octx, okeys, kvl, x, oxc, reduce=False)
    elif index:
        qk = lambda x: vmm.qk_scores_indexed(ops, kvl, x, oxc, replicate=False)
    oms = vmm.gqa_qk_scores(ops, glay, oq, okc, masks, opts(0, lv + 1), qk=qk)
    gms = gctx.gqa_qk(gkeys, gqa, gq)
    assert len(gms) == G
    for om, gm in zip(oms, gms):
        _same(e, om, gm)
    got = glay.unpack_scores([gctx.decrypt(e["gsk"], gm).real for gm in gms], ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, np.repeat(K, G, axis=1))).max() < TOL
    pairs = [_enc_both(e, v, lv, 50 + d) for d, v in enumerate(glay.pack_scores(s))]
    sv = (lambda c: vmm.score_times_v_unrolled(octx, okeys, kvl, c, ovc, reduce=False)) if unrolled else None
    oa = vmm.gqa_score_times_v(ops, glay, [p[0] for p in pairs], ovc, opts(1, lv - 1), sv=sv)
    ga = gctx.gqa_sv(gkeys, gqa, [p[1] for p in pairs])
    _same(e, oa, ga)
    att = glay.q.unpack_vec(gctx.decrypt(e["gsk"], ga).real)
    assert np.abs(att - np.einsum("hn,nhe->he", s, np.repeat(V, G, axis=1))).max() < TOL
    # errors: a query at the wrong level, a group that does not divide the block, a missing key
    with pytest.raises(B.CachemirError) as ei:
        gctx.gqa_qk(gkeys, gqa, gctx.level_drop(gq, lv))
    assert ei.value.status == -2
    with pytest.raises(B.CachemirError) as ei:
        gctx.gqa(kv, 128)
    assert ei.value.status == -5
    few = gctx.keygen_rotations(e["gsk"], [a for a in steps if a != gqa.steps()[0]], 2, with_relin=True)
    with pytest.raises(B.CachemirError) as ei:
        gctx.gqa_qk(few, gqa, gq)
    assert ei.value.status == -4


def test_twelve_heads_padded_to_sixteen_match_oracle_and_float64(env):
    """GPT2-base head count on the small ring (12 heads of 64 dims -> 16 x 64, t = 2): appends, q K^T and scores V
    limb for limb against the oracle with the padded layout, values against the einsum over the 12 real heads."""
    from oracle import packing, vmm
    from oracle.ckks import Pt
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    H, E, ntok, L = 12, 64, 7, octx.prm.L
    lay = packing.KvLayout(octx.S, H, E, 8)
    assert (lay.H, lay.t) == (16, 2)
    rng = np.random.default_rng(12)
    q = rng.normal(size=(H, E)) * 0.3
    K, V = rng.normal(size=(ntok, H, E)), rng.normal(size=(ntok, H, E))
    s = rng.uniform(0, 1, size=(H, ntok))
    s /= s.sum(axis=1, keepdims=True)
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, r_i=8)
    steps = lay.qk_steps() + lay.sv_steps() + lay.append_steps()
    assert sorted(set(kv.steps())) == sorted(set(steps))
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    ops = vmm.CkksOps(octx, okeys)

    def base(kind, level):
        m = np.zeros(octx.S)
        if kind == 0:
            m[:lay.H * lay.t] = 1
        elif kind == 1:
            m[::lay.t] = 1
        else:
            m[[h * lay.t for h in range(lay.H)]] = 1
        return octx.encode_coeffs(m, float(octx.mod[level]))
    bases = {0: base(0, lv - 1), 1: base(1, lv + 1), 2: base(2, lv + 1)}
    for kind, c in bases.items():
        kv.set_mask(kind, c)

    def omask(kind, shift_right, level):
        idx = octx.q_idx(level)
        coeff = octx.automorphism_coeff(octx.from_i64(bases[kind], idx), idx, octx.galois(-shift_right))
        return Pt(octx.ntt(coeff, idx), level, float(octx.mod[level]))
    okc, ovc = [], [None] * E
    for n in range(ntok):
        c, tau = n // lay.t, n % lay.t
        ok_new, gk_new = _enc_both(e, lay.pack_vec(K[n], tau), L, 100 + n)
        ov_new, gv_new = _enc_both(e, lay.pack_vec(V[n], tau), L, 500 + n)
        vmasks = [omask(2, lay.slot((c - k) % E, 0, tau) + lay.v_shift(k), lv + 1) for k in range(E)]
        vmm.kv_append(ops, lay, okc, ovc, n, ok_new, ov_new, omask(1, tau, lv + 1), vmasks)
        kv.append(gkeys, gk_new, gv_new)
    for c in range(len(okc)):
        assert np.array_equal(kv.export(B.CM_QK, c), octx.canonical(okc[c]))
    for k in (0, 5, E - 1):
        assert np.array_equal(kv.export(B.CM_SV, k), octx.canonical(ovc[k]))
    oq, gq = _enc_both(e, lay.pack_vec(q), lv, 10)
    om = vmm.qk_scores(ops, lay, oq, okc, [omask(0, (c % E) * lay.H * lay.t, lv - 1) for c in range(len(okc))])
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
    _same(e, om, gm)
    assert np.abs(lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok) - np.einsum("he,nhe->hn", q, K)).max() < TOL
    os_, gs = _enc_both(e, lay.pack_scores(s), lv, 50)
    oa = vmm.score_times_v(ops, lay, os_, ovc)
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
    _same(e, oa, ga)
    assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


@pytest.fixture(scope="module")
def ring2():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2602_11470_amd import binding as B
    gctx = B.llama_ring(24, 4)
    yield B, gctx
    gctx.close()


def test_config3_at_its_stated_size_with_every_kv_head_stored_once(ring2):
    """Benchmark configuration 3 as stated: 32 query heads x 128 dims, 8 KV heads, context 1024, on the 24 + 4
    ring.  The cache holds the 8 KV heads once: 32 K ciphertexts of 32 tokens and 128 V ciphertexts (a quarter of
    the replicated layout's 128 + 128 per 1024 tokens at four times the capacity).  q K^T in four passes, scores
    V in four passes, against float64; the k projection's natural layout (a contracting 4096 -> 1024 product)
    feeds the append of token 1024."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    B, gctx = ring2
    H, Hkv, E, ntok, L = 32, 8, 128, 1024, gctx.L
    glay = packing.GqaLayout(gctx.S, H, Hkv, E, 16)
    kvl, G = glay.kv, glay.G
    assert (kvl.t, glay.t, kvl.capacity, G) == (32, 8, 4096, 4)
    rng = np.random.default_rng(3)
    q = rng.normal(size=(H, E))
    K, V = rng.normal(size=(ntok + 1, Hkv, E)), rng.normal(size=(ntok + 1, Hkv, E))
    s = rng.uniform(0, 1, size=(H, ntok + 1))
    s /= s.sum(axis=1, keepdims=True)
    lv = L - 2
    kv = gctx.kv_create(Hkv, E, lv, r_i=16, unrolled_ladders=True, shared_dims=32)
    gqa = gctx.gqa(kv, G)
    gsk = gctx.keygen_secret(1)
    steps = sorted({a for a in kv.steps() if a % kvl.t == 0} | set(gqa.steps()))
    gkeys = gctx.keygen_rotations(gsk, steps, 2, with_relin=True)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, L), seed), level)
    nk = ntok // kvl.t
    for c in range(nk):
        kv.load(B.CM_QK, c, enc(kvl.pack_k(K[:ntok], c), lv, 100 + c))
    for k in range(E):
        kv.load(B.CM_SV, k, enc(kvl.pack_v(V[:ntok], k), lv, 300 + k))
    kv.set_tokens(ntok)
    # token 1024 arrives the way a contracting k / v projection leaves it: element e*Hkv + hk at slot (e*Hkv + hk)*32 + tau
    tau = ntok % kvl.t
    kv.append(gkeys, enc(kvl.pack_vec(K[ntok], tau), lv + 1, 600), enc(kvl.pack_vec(V[ntok], tau), lv + 1, 601))
    assert kv.tokens() == ntok + 1
    gms = gctx.gqa_qk(gkeys, gqa, enc(glay.q.pack_vec(q), lv + 1, 10))
    assert all(gm.level == lv - 2 for gm in gms)
    got = glay.unpack_scores([gctx.decrypt(gsk, gm).real for gm in gms], ntok + 1)
    assert np.abs(got - np.einsum("he,nhe->hn", q, np.repeat(K, G, axis=1))).max() < TOL
    ga = gctx.gqa_sv(gkeys, gqa, [enc(v, lv, 50 + d) for d, v in enumerate(glay.pack_scores(s))])
    assert ga.level == lv - 2
    att = glay.q.unpack_vec(gctx.decrypt(gsk, ga).real)
    assert np.abs(att - np.einsum("hn,nhe->he", s, np.repeat(V, G, axis=1))).max() < TOL


def test_gpt2_base_attention_shape_on_the_full_ring(ring2):
    """12 heads of 64 dims (Table 3) on 2^15 slots: padded to 16 heads, t = 32 tokens per K ciphertext, 64 V
    ciphertexts; 70 tokens by loads and three appends; q K^T and scores V against float64."""
    from oracle import packing
    B, gctx = ring2
    H, E, L = 12, 64, gctx.L
    lay = packing.KvLayout(gctx.S, H, E, 8)
    assert (lay.H, lay.t, lay.capacity) == (16, 32, 2048)
    n_loaded, n_app = 67, 3
    ntok = n_loaded + n_app
    rng = np.random.default_rng(13)
    q = rng.normal(size=(H, E))
    K, V = rng.normal(size=(ntok, H, E)), rng.normal(size=(ntok, H, E))
    s = rng.uniform(0, 1, size=(H, ntok))
    s /= s.sum(axis=1, keepdims=True)
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, r_i=8, unrolled_ladders=True, shared_dims=16)
    gsk = gctx.keygen_secret(1)
    gkeys = gctx.keygen_rotations(gsk, kv.steps(), 2, with_relin=True)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, L), seed), level)
    for c in range(-(-n_loaded // lay.t)):
        kv.load(B.CM_QK, c, enc(lay.pack_k(K[:n_loaded], c), lv, 100 + c))
    for k in range(E):
        kv.load(B.CM_SV, k, enc(lay.pack_v(V[:n_loaded], k), lv, 300 + k))
    kv.set_tokens(n_loaded)
    for n in range(n_loaded, ntok):
        tau = n % lay.t
        kv.append(gkeys, enc(lay.pack_vec(K[n], tau), L, 600 + n), enc(lay.pack_vec(V[n], tau), L, 700 + n))
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, enc(lay.pack_vec(q), lv, 10))
    assert np.abs(lay.unpack_scores(gctx.decrypt(gsk, gm).real, ntok) - np.einsum("he,nhe->hn", q, K)).max() < TOL
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, enc(lay.pack_scores(s), lv, 50))
    assert np.abs(lay.unpack_vec(gctx.decrypt(gsk, ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL
