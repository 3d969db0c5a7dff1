"""GPU parity at the benchmark's full sizes (ring n = 2^16), in the launch configuration bench.py
times: single operations element by element against the oracle, the full 4096x4096 packed
product against a stored oracle result, and the decrypted product against float64."""
import hashlib

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _llama(n_q, n_p):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import ckks, params
    from paper_2602_11470_amd import binding as B
    prm = params.llama_ring(n_q, n_p)
    return B, ckks.Context(prm), B.llama_ring(n_q, n_p), prm


@pytest.fixture(scope="module")
def ring2():
    B, octx, gctx, prm = _llama(24, 4)
    yield B, octx, gctx, prm
    gctx.close()


def _pair(octx, gctx, osk, gsk, coeffs, level, seed):
    scale = octx.prm.scale
    o = octx.encrypt(osk, octx.pt_from_coeffs(coeffs, level, scale), seed)
    g = gctx.encrypt(gsk, gctx.pt_from_coeffs(coeffs, level, scale), seed)
    return o, g


def test_config2_chain_keys_and_single_operations(ring2):
    B, octx, gctx, prm = ring2
    assert gctx.moduli().tolist() == prm.moduli
    osk, gsk = octx.keygen_secret(1), gctx.keygen_secret(1)
    assert np.array_equal(gsk.coeffs().astype(np.int64), osk["coeffs"])
    assert int((osk["coeffs"] != 0).sum()) == 192
    steps = [7, 2048]
    okeys = octx.keygen_rotations(osk, steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(gsk, steps, 2, with_relin=True)
    all_idx = list(range(len(octx.mod)))
    g7 = octx.galois(7)
    assert np.array_equal(gkeys.export(7, False, 5, 0), octx.intt(okeys[g7].b[5], all_idx))
    assert np.array_equal(gkeys.export(7, False, 0, 1), octx.intt(okeys[g7].a[0], all_idx))
    rng = np.random.default_rng(0)
    z = rng.normal(size=octx.S)
    coeffs = octx.encode_coeffs(z, prm.scale)
    o, g = _pair(octx, gctx, osk, gsk, coeffs, prm.L, 3)
    assert np.array_equal(gctx.ct_export(g), octx.canonical(o))
    # full key switch at the top level (24 limbs, 6 digits of 4 primes, 4 special primes)
    orot, grot = octx.rotate(o, 7, okeys), gctx.rotate(gkeys, g, 7)
    assert np.array_equal(gctx.ct_export(grot), octx.canonical(orot))
    assert np.abs(gctx.decrypt(gsk, grot).real - np.roll(z, -7)).max() < 1e-6
    # hoisted rotations
    h = octx.hoist(o)
    for s, gout in zip(steps, gctx.rotate_hoisted(gkeys, g, steps)):
        assert np.array_equal(gctx.ct_export(gout), octx.canonical(octx.rotate_hoisted(o, h, s, okeys)))
    # a partial last digit (level 4: digits of 4 + 1 primes), product, relinearisation, rescale
    o4, g4 = octx.level_drop(o, 4), gctx.level_drop(g, 4)
    assert np.array_equal(gctx.ct_export(gctx.rotate(gkeys, g4, 2048)), octx.canonical(octx.rotate(o4, 2048, okeys)))
    om = octx.rescale(octx.relinearize(octx.mul_ct(o4, o4), okeys))
    gm = gctx.rescale(gctx.relinearize(gkeys, gctx.mul_ct(g4, g4)))
    assert np.array_equal(gctx.ct_export(gm), octx.canonical(om))
    assert np.abs(gctx.decrypt(gsk, gm).real - z * z).max() < 1e-6


@pytest.mark.parametrize("form", ["plain", "raised", "direct", "unrolled", "mlp_up", "mlp_down"])
def test_config2_full_packed_product_against_stored_oracle_result(ring2, golden, form):
    """52 rotations (84 in the unrolled form with its 64 x 8 split), 512 plaintext multiply-accumulates at (S, d) =
    (32768, 4096); the expected ciphertext was written by tests/golden/make_vmm_full_size_golden.py
    from the oracle, for the algorithm as printed, for the form that keeps the baby-step sums in the
    extended basis, for that with the giant steps unrolled, and for that with the two ladders
    unrolled as well (the configuration bench.py times).  mlp_up / mlp_down: the MLP shapes of benchmark
    configuration 4 (4096 -> 16384 and back, 14336 padded; 2048 products, 128 x 16 steps, 150 rotations) at the
    paper's operating level 4, unrolled form."""
    import importlib.util
    import os
    B, octx, gctx, prm = ring2
    mlp = form.startswith("mlp")
    raised, direct, unrolled = form != "plain", form == "direct", form == "unrolled" or mlp
    g = golden({"plain": "vmm_full_size.txt", "raised": "vmm_full_size_raised.txt", "direct": "vmm_full_size_direct.txt",
                "unrolled": "vmm_full_size_unrolled.txt", "mlp_up": "vmm_full_size_mlp_up.txt",
                "mlp_down": "vmm_full_size_mlp_down.txt"}[form])
    spec = importlib.util.spec_from_file_location(
        "mk", os.path.join(os.path.dirname(__file__), "golden", "make_vmm_full_size_golden.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    plan = mk.plan_for(octx.S, form)
    level = mk.level_for(prm, form)
    xc, diag = mk.integer_inputs(octx.n, plan)
    gplan = gctx.vmm_plan(plan.d_in, plan.d_out, level=level, r_i=plan.r_i, coeffs=np.stack(diag), pt_scale=prm.scale,
                          raised_sums=raised, direct_giants=direct, unrolled_ladders=unrolled)
    del diag
    assert gplan.n_rotations == int(g["rotations"]) == (150 if mlp else 84 if unrolled else 52)
    assert (gplan.r_i, gplan.r_o) == ((128, 16) if mlp else (64, 8) if unrolled else (32, 16))
    assert gplan.r_i * gplan.r_o == int(g["pt_mults"]) == (2048 if mlp else 512)
    gsk = gctx.keygen_secret(mk.SEED_SK)
    gkeys = gctx.keygen_rotations(gsk, gplan.steps(), mk.SEED_EVK)
    gx = gctx.level_drop(gctx.encrypt(gsk, gctx.pt_from_coeffs(xc, prm.L, prm.scale), mk.SEED_ENC), level)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    can = gctx.ct_export(gy)
    assert list(can.shape) == [int(v) for v in g["shape"].split()] and gy.level == int(g["level"])
    for c in range(can.shape[0]):
        for l in range(can.shape[1]):
            assert [int(v) for v in can[c, l, :4]] == [int(v) for v in g[f"head_{c}_{l}"].split()], (c, l)
    assert hashlib.sha256(can.tobytes()).hexdigest() == g["sha256"]


def test_config2_packed_product_decrypts_to_float64_product(ring2):
    from paper_2602_11470_amd import inputs
    B, octx, gctx, prm = ring2
    d = 4096
    x, W = inputs.vmm_inputs(1, d, d)
    gplan = gctx.vmm_plan(d, d, W=W)
    gsk = gctx.keygen_secret(1)
    gkeys = gctx.keygen_rotations(gsk, gplan.steps(), 2)
    t = gctx.S // d
    slots = np.zeros(gctx.S)
    slots[::t] = x
    gx = gctx.encrypt(gsk, gctx.encode(slots, gctx.L), 3)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    out = gctx.decrypt(gsk, gy)
    assert np.abs(out.real[::t] - x @ W).max() < TOL
    assert gy.level == gctx.L - 1
    r_i = gplan.r_i
    del gplan
    # baby-step sums kept in the extended basis (same split, same keys): the same message up to rounding noise
    gplan_r = gctx.vmm_plan(d, d, W=W, raised_sums=True, r_i=r_i)
    gyr = gctx.vmm_pt(gkeys, gplan_r, gx)
    assert gyr.level == gy.level and abs(gyr.scale / gy.scale - 1) < 1e-12
    outr = gctx.decrypt(gsk, gyr)
    assert np.abs(outr.real[::t] - x @ W).max() < TOL and np.abs(outr - out).max() < 1e-6
    del gplan_r
    # the operating level of the paper's projections (level 4): two digits, the last one partial
    gplan4 = gctx.vmm_plan(d, d, W=W, level=4)
    gx4 = gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, gctx.L), 3), 4)
    out4 = gctx.decrypt(gsk, gctx.vmm_pt(gkeys, gplan4, gx4))
    assert np.abs(out4.real[::t] - x @ W).max() < TOL


@pytest.mark.parametrize("d,level,rotations", [
    (2048, 23, 30),      # TinyLlama-1.1B width (Table 4: 30 rotations)
    (1024, 23, 20),      # GPT2-base width 768 padded to 1024 (Table 4: 20 rotations)
    (4096, 13, 52),      # the paper's starting level
    (4096, 1, 52),       # lowest level a product can run at (one digit, partial)
])
def test_other_widths_and_levels_decrypt_to_float64_product(ring2, d, level, rotations):
    """Square projections of the paper's other models and of its level sweep on the full ring, in
    the form bench.py times (raised sums, unrolled giant steps)."""
    from paper_2602_11470_amd import inputs
    B, octx, gctx, prm = ring2
    x, W = inputs.vmm_inputs(7, d, d)
    if d == 1024:                      # a 768-wide layer zero-padded to the next power of two
        x[768:] = 0.0
        W[768:, :] = 0.0
        W[:, 768:] = 0.0
    from oracle import packing
    plan = packing.make_plan(octx.S, d, d)
    assert plan.n_rotations == rotations                       # as Algorithm 1 counts them with the square-root split
    gplan = gctx.vmm_plan(d, d, W=W, level=level, unrolled_ladders=True)
    assert (gplan.r_i, gplan.r_o) == (2 * plan.r_i, plan.r_o // 2)     # the library doubles the cheap baby steps
    gsk = gctx.keygen_secret(1)
    gkeys = gctx.keygen_rotations(gsk, gplan.steps(), 2)
    t = gctx.S // d
    slots = np.zeros(gctx.S)
    slots[::t] = x
    gx = gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, gctx.L), 3), level)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    assert gy.level == level - 1
    out = gctx.decrypt(gsk, gy)
    assert np.abs(out.real[::t] - x @ W).max() < TOL


@pytest.mark.parametrize("d_in,d_out", [(4096, 16384), (16384, 4096)])
def test_config4_mlp_projection_shapes_decrypt_to_float64_product(ring2, d_in, d_out):
    """The MLP projections of Llama-3-8B (4096 -> 14336 -> 4096) with the long side zero-padded to
    16384 = 4 x 4096: 2048 weight diagonals (64 baby x 32 giant steps), 98 rotations, at the paper's
    operating level 4, in the form bench.py times."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    B, octx, gctx, prm = ring2
    level, real = 4, 14336
    x, W = inputs.vmm_inputs(8, d_in, d_out)
    if d_in > d_out:
        x[real:] = 0.0
        W[real:, :] = 0.0
    else:
        W[:, real:] = 0.0
    plan = packing.make_plan(octx.S, d_in, d_out)
    gplan = gctx.vmm_plan(d_in, d_out, W=W, level=level, unrolled_ladders=True)
    assert (plan.r_i, plan.r_o, plan.n_rotations) == (64, 32, 98)
    assert (gplan.r_i, gplan.r_o) == (128, 16)                    # the library doubles the cheap baby steps
    assert gplan.n_rotations == 127 + 15 + (7 + 1)                # and the three-step ladder becomes seven hoisted rotations
    gsk = gctx.keygen_secret(1)
    gkeys = gctx.keygen_rotations(gsk, gplan.steps(), 2)
    gx = gctx.level_drop(gctx.encrypt(gsk, gctx.encode(plan.pack_input(x), gctx.L), 3), level)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    assert gy.level == level - 1
    out = plan.unpack_output(gctx.decrypt(gsk, gy).real)
    assert np.abs(out - x @ W).max() < TOL


@pytest.mark.parametrize("unrolled,shared,index", [(False, 1, False), (True, 1, False), (True, 128, False), (True, 16, False),
                                                   (True, 1, True)])
def test_config3_attention_shapes_decrypt_to_float64_products(ring2, unrolled, shared, index):
    """Llama-3-8B attention shapes on the full ring: 32 heads x 128 dims (8 KV heads repeated 4x),
    t = 8 tokens per K ciphertext, 128 V ciphertexts with 16 baby x 8 giant steps.  A short
    context (two loaded K ciphertexts plus three appended tokens) keeps the run small; every
    ciphertext and rotation has its full size.  shared > 1: the copy mask before the last `shared`
    terms of the sum over the dims (127 or 15 rotations for the whole cache); index: the cache keeps the
    key index, loaded for the first tokens and extended by the appends, and q K^T runs on it."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    B, octx, gctx, prm = ring2
    H, E, L = 32, 128, gctx.L
    lay = packing.KvLayout(gctx.S, H, E, 16)
    assert lay.t == 8 and lay.capacity == 1024
    n_loaded, n_app = 16, 3
    ntok = n_loaded + n_app
    q, K, V, s = inputs.attention_inputs(3, H, 8, E, ntok)
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, r_i=16, unrolled_ladders=unrolled, shared_dims=shared, key_index=index)
    gsk = gctx.keygen_secret(1)
    gkeys = gctx.keygen_rotations(gsk, kv.steps(), 2, with_relin=True)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, L), seed), level)
    for c in range(n_loaded // lay.t):
        kv.load(B.CM_QK, c, enc(lay.pack_k(K[:n_loaded], c), lv, 100 + c))
    for k in range(E):
        kv.load(B.CM_SV, k, enc(lay.pack_v(V[:n_loaded], k), lv, 300 + k))
        if index:
            kv.load(B.CM_KV_INDEX, k, enc(lay.pack_k_index(K[:n_loaded], k), lv, 800 + k))
    kv.set_tokens(n_loaded)
    for n in range(n_loaded, ntok):
        tau = n % lay.t
        kv.append(gkeys, enc(lay.pack_vec(K[n], tau), L, 600 + n), enc(lay.pack_vec(V[n], tau), L, 700 + n))
    assert kv.tokens() == ntok
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, enc(lay.pack_vec(q), lv, 10))
    assert gm.level == (lv - 1 if index else lv - 2)
    got = lay.unpack_scores(gctx.decrypt(gsk, gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, enc(lay.pack_scores(s), lv, 50))
    assert ga.level == lv - 1
    assert np.abs(lay.unpack_vec(gctx.decrypt(gsk, ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


@pytest.mark.parametrize("index", [False, True])
def test_prompt_phase_on_the_full_ring_builds_a_cache_the_decode_products_can_use(ring2, index):
    """Sec. 5.4 at Llama-3-8B shapes: two ciphertexts of t = 8 tokens each go through the token-batched
    4096 x 4096 k and v projections (4096 diagonals, 128 baby x 32 giant steps, columns ordered (e, h)),
    the rotary embedding of a token group and the group append; then the decode-phase q K^T and
    scores V run against that cache.  Everything is compared with the float64 computation.  index: the cache
    also keeps the key index, which the group appends extend and q K^T then runs on."""
    from oracle import packing
    B, octx, gctx, prm = ring2
    H, E, d = 32, 128, 4096
    lay = packing.KvLayout(gctx.S, H, E, 16)
    t, lvx = lay.t, 6
    lv = lvx - 3                                       # cache level: product, embedding, append mask
    rng = np.random.default_rng(21)
    groups = 2
    ntok = groups * t
    X = rng.uniform(-1, 1, size=(ntok, d))
    Wk, Wv = rng.uniform(-1, 1, size=(d, d)) / 64, rng.uniform(-1, 1, size=(d, d)) / 64
    gsk = gctx.keygen_secret(1)
    pk = gctx.vmm_plan(d, d, W=Wk, level=lvx, direct_giants=True, token_batch=True)
    pv = gctx.vmm_plan(d, d, W=Wv, level=lvx, direct_giants=True, token_batch=True)
    assert (pk.r_i, pk.r_o, pk.n_rotations) == (128, 32, 158)
    kv = gctx.kv_create(H, E, lv, r_i=16, key_index=index)
    ropes = [gctx.rope(H, E, lvx - 1, c * t, tau=-1) for c in range(groups)]
    steps = sorted(set(pk.steps()) | set(kv.steps()) | set(ropes[0].steps()))
    gkeys = gctx.keygen_rotations(gsk, steps, 2, with_relin=True)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, gctx.L), seed), level)
    for c in range(groups):
        Xc = X[c * t:(c + 1) * t]
        gx = enc(Xc.T.reshape(-1), lvx, 40 + c)                  # X[tau, b] at slot b t + tau
        gk, gv = gctx.vmm_pt_multi(gkeys, [pk, pv], gx)
        if c == 0:
            assert np.abs(gctx.decrypt(gsk, gk).real.reshape(d, t).T - Xc @ Wk).max() < TOL
        kv.append_group(gkeys, gctx.rope_apply(gkeys, ropes[c], gk), gctx.level_drop(gv, lvx - 2))
    assert kv.tokens() == ntok
    # float64 reference: column e*H + h of the products is element [h, e]
    K = (X @ Wk).reshape(ntok, E, H).transpose(0, 2, 1)
    V = (X @ Wv).reshape(ntok, E, H).transpose(0, 2, 1)
    Kr = np.empty_like(K)
    for n in range(ntok):
        for m in range(E // 2):
            th = n * 10000.0 ** (-2.0 * m / E)
            Kr[n, :, 2 * m] = K[n, :, 2 * m] * np.cos(th) - K[n, :, 2 * m + 1] * np.sin(th)
            Kr[n, :, 2 * m + 1] = K[n, :, 2 * m + 1] * np.cos(th) + K[n, :, 2 * m] * np.sin(th)
    q = rng.normal(size=(H, E)) * 0.3
    s = rng.uniform(0, 1, size=(H, ntok)) / ntok
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, enc(lay.pack_vec(q), lv, 10))
    got = lay.unpack_scores(gctx.decrypt(gsk, gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, Kr)).max() < TOL
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, enc(lay.pack_scores(s), lv, 50))
    assert np.abs(lay.unpack_vec(gctx.decrypt(gsk, ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


def test_prompt_phase_attention_of_a_query_group_on_the_full_ring(ring2):
    """Sec. 5.4 at Llama-3-8B attention shapes (32 heads x 128 dims, t = 8), extended-basis ladders: a
    group of 8 queries is inner-rotated by delta and meets two K ciphertexts without replication; the
    scores of a group meet V without the sum over the residues and are inner-rotated back by
    t - delta; the sum over the deltas taken is, per query, the float64 product of those scores with V."""
    from oracle import packing
    B, octx, gctx, prm = ring2
    H, E = 32, 128
    lay = packing.KvLayout(gctx.S, H, E, 16)
    t, nk = lay.t, 2
    ntok = nk * t
    lv = 5                                              # cache level; the query group arrives one level higher
    rng = np.random.default_rng(23)
    Q = rng.normal(size=(t, H, E)) * 0.3
    K = rng.normal(size=(ntok, H, E))
    V = rng.normal(size=(ntok, H, E))
    deltas = (0, 3)
    kv = gctx.kv_create(H, E, lv, r_i=16, unrolled_ladders=True)
    gsk = gctx.keygen_secret(1)
    rots = {d: (gctx.inner_rot(t, d, lv + 1), gctx.inner_rot(t, t - d, lv - 1)) for d in deltas if d}
    steps = {a for a in kv.steps() if a % t == 0}      # nothing moves a residue except the inner rotations
    for fwd, bwd in rots.values():
        steps |= set(fwd.steps()) | set(bwd.steps())
    gkeys = gctx.keygen_rotations(gsk, sorted(steps), 2, with_relin=True)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, gctx.L), seed), level)
    for c in range(nk):
        kv.load(B.CM_QK, c, enc(lay.pack_k(K, c), lv, 100 + c))
    for k in range(E):
        kv.load(B.CM_SV, k, enc(lay.pack_v(V, k), lv, 300 + k))
    kv.set_tokens(ntok)
    gq = enc(sum(lay.pack_vec(Q[tau], tau) for tau in range(t)), lv + 1, 10)
    full = np.einsum("ahe,nhe->ahn", Q, K)              # [query, head, key]
    out, want = None, np.zeros((t, H, E))
    for delta in deltas:
        gx = gctx.rope_apply(gkeys, rots[delta][0], gq) if delta else gctx.level_drop(gq, lv)
        gm = gctx.vmm_kv(gkeys, kv, B.CM_QK_GROUP, gx)
        got = lay.unpack_scores(gctx.decrypt(gsk, gm).real, ntok)
        for n in range(ntok):
            assert np.abs(got[:, n] - full[(n % t - delta) % t, :, n]).max() < TOL
        # scores of the group after the (plaintext-side) non-linearity: fresh values at the same slots
        s = rng.uniform(0, 1, size=(H, ntok)) / ntok
        ga = gctx.vmm_kv(gkeys, kv, B.CM_SV_GROUP, enc(lay.pack_scores(s), lv, 50 + delta))
        assert ga.level == lv - 1
        gb = gctx.rope_apply(gkeys, rots[delta][1], ga) if delta else gctx.level_drop(ga, lv - 2)
        out = gb if out is None else gctx.add(out, gb)
        for n in range(ntok):                           # s[h, n] belongs to query (n % t - delta) mod t
            want[(n % t - delta) % t] += s[:, n][:, None] * V[n]
    res = gctx.decrypt(gsk, out).real
    for tau in range(t):
        assert np.abs(lay.unpack_vec(res, tau) - want[tau]).max() < TOL


def test_appends_with_the_masked_product_inside_the_rescale_equal_the_two_step_appends(ring2):
    """At n = 2^16 an append forms its masked products inside the tail of the rescale's transform; with the
    context option CM_OPT_TWO_STEP_MASKS it multiplies, stores and rescales (the path the small-ring tests
    check limb for limb against the oracle).  Same cache, same key index, bit for bit: one token group and
    two single tokens."""
    from oracle import packing
    B, octx, gctx, prm = ring2
    H, E, lv = 32, 128, 4
    lay = packing.KvLayout(gctx.S, H, E, 16)
    rng = np.random.default_rng(77)
    gsk = gctx.keygen_secret(1)
    enc = lambda slots, level, seed: gctx.level_drop(gctx.encrypt(gsk, gctx.encode(slots, gctx.L), seed), level)
    news = [(enc(rng.normal(size=gctx.S), lv + 1, 900 + 2 * i), enc(rng.normal(size=gctx.S), lv + 1, 901 + 2 * i)) for i in range(3)]
    caches = []
    keys = None
    for two_step in (False, True):
        kv = gctx.kv_create(H, E, lv, r_i=16, key_index=True)
        if keys is None:
            keys = gctx.keygen_rotations(gsk, kv.steps(), 2, with_relin=True)
        gctx.set_option(B.CM_OPT_TWO_STEP_MASKS, two_step)
        try:
            kv.append_group(keys, *news[0])
            kv.append(keys, *news[1])
            kv.append(keys, *news[2])
        finally:
            gctx.set_option(B.CM_OPT_TWO_STEP_MASKS, False)
        caches.append(kv)
    a, b = caches
    assert a.tokens() == b.tokens() == lay.t + 2
    for k in (0, 1, 17, E - 1):
        assert np.array_equal(a.export(B.CM_SV, k), b.export(B.CM_SV, k)), k
        assert np.array_equal(a.export(B.CM_KV_INDEX, k), b.export(B.CM_KV_INDEX, k)), k
    assert np.array_equal(a.export(B.CM_QK, 0), b.export(B.CM_QK, 0))
    assert np.array_equal(a.export(B.CM_QK, 1), b.export(B.CM_QK, 1))


def test_config5_ring_rotation(ring2):
    """36 + 6 primes (6 digits of 6): one full key switch element by element."""
    B, octx, gctx, prm = _llama(36, 6)
    try:
        assert gctx.moduli().tolist() == prm.moduli
        osk, gsk = octx.keygen_secret(4), gctx.keygen_secret(4)
        okeys, gkeys = octx.keygen_rotations(osk, [256], 5), gctx.keygen_rotations(gsk, [256], 5)
        z = np.random.default_rng(1).normal(size=octx.S)
        o, g = _pair(octx, gctx, osk, gsk, octx.encode_coeffs(z, prm.scale), prm.L, 6)
        orot, grot = octx.rotate(o, 256, okeys), gctx.rotate(gkeys, g, 256)
        assert np.array_equal(gctx.ct_export(grot), octx.canonical(orot))
        assert np.abs(gctx.decrypt(gsk, grot).real - np.roll(z, -256)).max() < 1e-6
    finally:
        gctx.close()
