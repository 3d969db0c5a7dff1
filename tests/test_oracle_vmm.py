"""Oracle end to end: decrypted homomorphic products against the float64 products they stand
for (the result has a plain definition: y = x W, m = q K^T per head, Att = s V per head)."""
import numpy as np
import pytest

from oracle import ckks, packing, params, vmm
from paper_2602_11470_amd import inputs

TOL = 1e-4      # max-abs tolerance on decrypted results


def test_config1_vmm_decrypts_to_x_times_W():
    prm = params.config1()
    ctx = ckks.Context(prm)
    x, W = inputs.vmm_inputs(0, 64, 64, "uniform", 0.05)
    plan = packing.make_plan(ctx.S, 64, 64)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, plan.all_steps(), 2)
    assert len(keys) == 11
    ct = ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3)
    diags = [[ctx.encode(v, prm.L) for v in row] for row in plan.diagonals(W)]
    y = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, diags)
    assert (ctx.rot_count, ctx.ptmul_count) == (11, 2)
    assert y.level == prm.L - 1                      # depth 1
    out = ctx.decrypt(sk, y)
    assert np.abs(plan.unpack_output(out.real) - x @ W).max() < TOL
    assert np.abs(out.imag).max() < TOL


@pytest.mark.parametrize("d_in,d_out,level,tau", [(16, 16, 3, 0), (16, 64, 2, 0), (64, 16, 4, 0),
                                                  (32, 32, 1, 3)])
def test_small_ring_vmm_shapes_and_levels(d_in, d_out, level, tau):
    prm = params.toy(n=512, n_qi=4, n_p=2, alpha=2, hamming=32)
    ctx = ckks.Context(prm)
    x, W = inputs.vmm_inputs(5, d_in, d_out, "normal", 0.1)
    plan = packing.make_plan(ctx.S, d_in, d_out, tau=tau)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, plan.all_steps(), 2)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3), level)
    diags = [[ctx.encode(v, level) for v in row] for row in plan.diagonals(W)]
    y = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, diags)
    assert y.level == level - 1
    assert np.abs(plan.unpack_output(ctx.decrypt(sk, y).real) - x @ W).max() < TOL


@pytest.mark.parametrize("r_i", [0, 4])
def test_small_ring_attention_and_append(r_i):
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    lay = packing.KvLayout(ctx.S, 4, 8, r_i)
    ntok = lay.capacity - 3
    q, K, V, s = inputs.attention_inputs(2, 4, 2, 8, ntok)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, lay.qk_steps() + lay.sv_steps() + lay.append_steps(), 2,
                                with_relin=True)
    ops = vmm.CkksOps(ctx, keys)
    enc = lambda v, lv, seed: ctx.encrypt(sk, ctx.encode(v, lv), seed)
    # build the cache by appending token after token (inputs one level above the cache)
    kc, vc = [], [None] * lay.E
    for n in range(ntok):
        tau = n % lay.t
        vmm.kv_append(ops, lay, kc, vc, n, enc(lay.pack_vec(K[n], tau), L, 100 + n),
                      enc(lay.pack_vec(V[n], tau), L, 500 + n), lay.residue_mask(tau),
                      [lay.v_append_mask(k, n) for k in range(lay.E)])
    for c in (0, len(kc) - 1):
        assert np.abs(ctx.decrypt(sk, kc[c]).real - lay.pack_k(K, c)).max() < TOL
    for k in (0, lay.E - 1):
        assert np.abs(ctx.decrypt(sk, vc[k]).real - lay.pack_v(V, k)).max() < TOL
    cq = ctx.level_drop(enc(lay.pack_vec(q), L, 10), L - 1)
    m = vmm.qk_scores(ops, lay, cq, kc, [lay.qk_mask(c) for c in range(len(kc))])
    assert m.level == L - 3                            # depth 2 below the cache level
    got = lay.unpack_scores(ctx.decrypt(sk, m).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    cs = ctx.level_drop(enc(lay.pack_scores(s), L, 50), L - 1)
    a = vmm.score_times_v(ops, lay, cs, vc)
    assert a.level == L - 2
    assert np.abs(lay.unpack_vec(ctx.decrypt(sk, a).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


# ---- accumulation in the raised basis (double hoisting) -----------------------------------------
def _toy_ctx():
    prm = params.toy(n=512, n_qi=4, n_p=2, alpha=2, hamming=32)
    ctx = ckks.Context(prm)
    sk = ctx.keygen_secret(1)
    return prm, ctx, sk


def test_raised_rotation_divides_back_to_the_hoisted_rotation_exactly():
    """ModDown(u + P a) = ModDown(u) + a limb for limb (P a vanishes on the special limbs), so the
    raised forms must reproduce the ordinary operations bit for bit."""
    prm, ctx, sk = _toy_ctx()
    keys = ctx.keygen_rotations(sk, [3, 20], 2)
    z = np.random.default_rng(0).normal(size=ctx.S)
    for level in (prm.L, 2):
        x = ctx.level_drop(ctx.encrypt(sk, ctx.encode(z, prm.L), 3), level)
        back = ctx.moddown_ct(ctx.raise_ct(x), level, x.scale)
        assert all(np.array_equal(a, b) for a, b in zip(back.c, x.c))
        h = ctx.hoist(x)
        for r in (3, 20):
            want = ctx.rotate_hoisted(x, h, r, keys)
            got = ctx.moddown_ct(ctx.rotate_hoisted_raised(x, h, r, keys), level, x.scale)
            assert all(np.array_equal(a, b) for a, b in zip(got.c, want.c))
        zero = [np.zeros((len(ctx.ext_idx(level)), ctx.n), dtype=np.uint64) for _ in range(2)]
        want = ctx.rotate(x, 3, keys)
        got = ctx.rotate_add_raised(x, 3, keys, zero)
        assert all(np.array_equal(a, b) for a, b in zip(got.c, want.c))


def test_rotate_add_raised_is_rotation_plus_the_divided_addend():
    """Rot(x, r) + ModDown(E) against the two done separately.  ModDown(u) = floor(u / P) - a with
    a in [0, K) from the uncorrected base conversion, so the two differ per coefficient by one
    carry and three such terms, at most 2K - 1 in size; they agree after decryption."""
    prm, ctx, sk = _toy_ctx()
    keys = ctx.keygen_rotations(sk, [3, 5], 2)
    rng = np.random.default_rng(1)
    z, w, v = rng.normal(size=(3, ctx.S))
    level = prm.L
    x = ctx.encrypt(sk, ctx.encode(z, level), 3)
    y = ctx.encrypt(sk, ctx.encode(w, level), 4)
    E = ctx.rotate_hoisted_raised(y, ctx.hoist(y), 5, keys)
    got = ctx.rotate_add_raised(x, 3, keys, E)
    want = ctx.ct_add(ctx.rotate(x, 3, keys), ctx.moddown_ct(E, level, y.scale))
    a, b = ctx.canonical(got).astype(np.int64), ctx.canonical(want).astype(np.int64)
    q = np.array(prm.moduli[:level + 1], dtype=np.int64)[None, :, None]
    diff = (a - b) % q
    diff = np.minimum(diff, q - diff)
    assert 1 <= diff.max() <= 2 * prm.K - 1             # additive up to the rounding, and not identical
    assert np.abs(ctx.decrypt(sk, got).real - (np.roll(z, -3) + np.roll(w, -5))).max() < 1e-6
    # plaintext product in the raised basis: ModDown(R * p) decrypts to slots * p
    pt = ctx.encode_ext(v, level)
    acc = [np.zeros_like(E[0]), np.zeros_like(E[1])]
    ctx.mac_pt_raised(acc, E, pt, level)
    prod = ctx.rescale(ctx.moddown_ct(acc, level, y.scale * pt.scale))
    assert np.abs(ctx.decrypt(sk, prod).real - np.roll(w, -5) * v).max() < 1e-6
    assert np.array_equal(pt.m[:level + 1], ctx.encode(v, level).m)   # same polynomial on the q limbs


def test_rotation_inside_the_raised_basis():
    """rotate_raised: exact where exactness is forced (a raised ciphertext P ct vanishes on the
    special limbs, so nothing is lost by not dividing its first component), and within the
    rounding of one ModDown otherwise: second component identical, first within 2K."""
    prm, ctx, sk = _toy_ctx()
    keys = ctx.keygen_rotations(sk, [3, 5], 2)
    rng = np.random.default_rng(2)
    z, w = rng.normal(size=(2, ctx.S))
    for level in (prm.L, 2):
        x = ctx.level_drop(ctx.encrypt(sk, ctx.encode(z, prm.L), 3), level)
        got = ctx.rotate_raised(ctx.raise_ct(x), level, 3, keys)
        want = ctx.rotate_hoisted_raised(x, ctx.hoist(x), 3, keys)
        assert all(np.array_equal(a, b) for a, b in zip(got, want))
        # a raised sum with full special limbs: a hoisted rotation of another ciphertext times a plaintext
        y = ctx.level_drop(ctx.encrypt(sk, ctx.encode(w, prm.L), 4), level)
        R = [np.zeros((len(ctx.ext_idx(level)), ctx.n), dtype=np.uint64) for _ in range(2)]
        ctx.mac_pt_raised(R, ctx.rotate_hoisted_raised(y, ctx.hoist(y), 5, keys), ctx.encode_ext(z, level), level)
        assert R[0][level + 1:].any()
        scale = y.scale * prm.scale
        got = ctx.moddown_ct(ctx.rotate_raised(R, level, 3, keys), level, scale)
        down = ctx.moddown_ct(R, level, scale)
        want = ctx.rotate_hoisted(down, ctx.hoist(down), 3, keys)        # Galois map after the raise, as here
        assert np.array_equal(got.c[1], want.c[1])
        q = np.array(prm.moduli[:level + 1], dtype=np.int64)[:, None]
        diff = (got.c[0].astype(np.int64) - want.c[0].astype(np.int64)) % q
        # evaluation-domain limbs: compare coefficients
        dc = (ctx.intt(got.c[0], ctx.q_idx(level)).astype(np.int64) - ctx.intt(want.c[0], ctx.q_idx(level)).astype(np.int64)) % q
        dc = np.minimum(dc, q - dc)
        assert diff.any() and 1 <= dc.max() <= 2 * prm.K
        m = ctx.decrypt(sk, ctx.rescale(got)).real
        assert np.abs(m - np.roll(np.roll(w, -5) * z, -3)).max() < 1e-6


@pytest.mark.parametrize("d_in,d_out,level,tau", [(16, 16, 3, 0), (16, 64, 2, 0), (64, 16, 4, 0), (32, 32, 1, 3)])
def test_double_hoisted_vmm_decrypts_to_x_times_W(d_in, d_out, level, tau):
    prm, ctx, sk = _toy_ctx()
    x, W = inputs.vmm_inputs(5, d_in, d_out, "normal", 0.1)
    plan = packing.make_plan(ctx.S, d_in, d_out, tau=tau)
    keys = ctx.keygen_rotations(sk, plan.all_steps(), 2)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3), level)
    diags = plan.diagonals(W)
    ext = [[ctx.encode_ext(v, level) for v in row] for row in diags]
    r0, p0 = ctx.rot_count, ctx.ptmul_count
    y = vmm.vmm_pt_double_hoisted(ctx, keys, plan, ct, ext)
    assert ctx.rot_count - r0 == plan.n_rotations and ctx.ptmul_count - p0 == plan.r_i * plan.r_o
    assert y.level == level - 1
    got = plan.unpack_output(ctx.decrypt(sk, y).real)
    assert np.abs(got - x @ W).max() < TOL
    # against the plain algorithm: same message, limbs differ only by rounding noise
    plain = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, [[ctx.encode(v, level) for v in row] for row in diags])
    assert abs(y.scale / plain.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, y) - ctx.decrypt(sk, plain)).max() < 1e-6


@pytest.mark.parametrize("d_in,d_out,level,tau", [(64, 64, 3, 0), (16, 64, 2, 0), (64, 16, 4, 0), (32, 32, 1, 3)])
def test_direct_giant_steps_vmm_decrypts_to_x_times_W(d_in, d_out, level, tau):
    """Giant steps unrolled (independent rotations by k G, one shared ModDown): same rotation and
    product counts, same message as the nested form."""
    prm, ctx, sk = _toy_ctx()
    x, W = inputs.vmm_inputs(6, d_in, d_out, "normal", 0.1)
    plan = packing.make_plan(ctx.S, d_in, d_out, tau=tau)
    assert plan.r_o >= 2
    steps = vmm.direct_giant_steps(plan)
    assert len(steps) == plan.n_rotations
    keys = ctx.keygen_rotations(sk, sorted(set(steps) | set(plan.all_steps())), 2)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3), level)
    ext = [[ctx.encode_ext(v, level) for v in row] for row in plan.diagonals(W)]
    r0, p0 = ctx.rot_count, ctx.ptmul_count
    y = vmm.vmm_pt_direct_giants(ctx, keys, plan, ct, ext)
    assert ctx.rot_count - r0 == plan.n_rotations and ctx.ptmul_count - p0 == plan.r_i * plan.r_o
    assert y.level == level - 1
    assert np.abs(plan.unpack_output(ctx.decrypt(sk, y).real) - x @ W).max() < TOL
    nested = vmm.vmm_pt_double_hoisted(ctx, keys, plan, ct, ext)
    assert abs(y.scale / nested.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, y) - ctx.decrypt(sk, nested)).max() < 1e-6
    assert not np.array_equal(ctx.canonical(y), ctx.canonical(nested))     # different noise, same message


# ---- rotary embedding with fused extraction (Sec. 4.2, App. D) -------------------------------------
def _rope_reference(v, n, base=10000.0):
    """Textbook rotary embedding on v[h, e]: each pair (2m, 2m+1) turned by n * base^(-2m/E)."""
    H, E = v.shape
    out = np.empty_like(v)
    for m in range(E // 2):
        th = n * base ** (-2.0 * m / E)
        c, s_ = np.cos(th), np.sin(th)
        out[:, 2 * m] = v[:, 2 * m] * c - v[:, 2 * m + 1] * s_
        out[:, 2 * m + 1] = v[:, 2 * m + 1] * c + v[:, 2 * m] * s_
    return out


@pytest.mark.parametrize("tau,n", [(0, 0), (0, 5), (3, 1234)])
def test_rope_on_slots_is_the_textbook_rotation_and_cleans_other_slots(tau, n):
    lay = packing.KvLayout(512, 4, 8)          # t = 16
    rng = np.random.default_rng(n)
    v = rng.normal(size=(4, 8))
    slots = rng.normal(size=512)               # garbage everywhere (partial sums of a product) ...
    for h in range(4):
        for e in range(8):
            slots[lay.slot(e, h, tau)] = v[h, e]   # ... except the valid slots
    ops = vmm.SlotOps()
    out = vmm.rope(ops, lay, slots, lay.rope_plaintexts(n, tau))
    assert (ops.rotations, ops.pt_mults) == (2, 3)
    want = _rope_reference(v, n)
    assert np.abs(lay.unpack_vec(out, tau) - want).max() < 1e-12
    valid = np.zeros(512, dtype=bool)
    valid[[lay.slot(e, h, tau) for e in range(8) for h in range(4)]] = True
    assert np.abs(out[~valid]).max() == 0.0
    # norms of the pairs are kept (a rotation), and n = 0 is the identity on the valid slots
    assert np.allclose((want ** 2).reshape(4, 4, 2).sum(-1), (v ** 2).reshape(4, 4, 2).sum(-1))
    if n == 0:
        assert np.abs(lay.unpack_vec(out, tau) - v).max() == 0.0


def test_rope_on_ciphertexts_decrypts_to_the_rotation():
    prm = params.toy(n=512, n_qi=3, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    lay = packing.KvLayout(ctx.S, 4, 8)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, [lay.rope_step, -lay.rope_step], 2)
    rng = np.random.default_rng(3)
    v = rng.normal(size=(4, 8))
    slots = rng.normal(size=ctx.S)
    for h in range(4):
        for e in range(8):
            slots[lay.slot(e, h, 2)] = v[h, e]
    ct = ctx.encrypt(sk, ctx.encode(slots, prm.L), 3)
    # plaintexts at the scale of the prime the rescale removes: the ciphertext scale is unchanged
    ops = vmm.CkksOps(ctx, keys, pt_scale=float(prm.moduli[prm.L]))
    y = vmm.rope(ops, lay, ct, lay.rope_plaintexts(77, 2))
    assert y.level == prm.L - 1 and abs(y.scale / ct.scale - 1) < 1e-12
    out = ctx.decrypt(sk, y).real
    assert np.abs(lay.unpack_vec(out, 2) - _rope_reference(v, 77)).max() < 1e-6
    assert np.abs(out).max() < 10 and np.abs(out[1::lay.t]).max() < 1e-6      # residue 1 was garbage, now clean


# ---- the prompt phase (Sec. 5.4): t tokens per ciphertext, cache generation by token group ----------
@pytest.mark.parametrize("d,r_i", [(16, None), (16, 1), (16, 16), (64, None), (8, 2)])
def test_token_batched_product_on_slots_is_X_times_W(d, r_i):
    """Every residue of a block carries its own token, so one product gives the t rows of X W;
    r_i + r_o - 2 block rotations, d plaintext products, nothing else."""
    S = 128
    plan = packing.make_plan(S, d, d, r_i=r_i, tokens=True)
    assert plan.pre_steps == [] and plan.reduce_steps == [] and plan.M == d and plan.t == S // d
    assert all(s % plan.t == 0 for s in plan.all_steps())          # whole blocks only
    rng = np.random.default_rng(d)
    X, W = rng.normal(size=(plan.t, d)), rng.normal(size=(d, d))
    ops = vmm.SlotOps()
    y = vmm.vmm_pt(ops, plan, plan.pack_tokens(X), plan.diagonals(W))
    assert np.abs(plan.unpack_tokens(y) - X @ W).max() < 1e-12
    assert ops.rotations == plan.r_i + plan.r_o - 2 and ops.pt_mults == d
    # layout: token tau of element b at slot b*t + tau
    assert plan.pack_tokens(X)[5 * plan.t + 1] == X[1, 5]
    # a permutation matrix moves blocks and leaves the residues alone
    P = np.roll(np.eye(d), 3, axis=1)                               # y[c] = x[c - 3]
    y = vmm.vmm_pt(vmm.SlotOps(), plan, plan.pack_tokens(X), plan.diagonals(P))
    assert np.array_equal(plan.unpack_tokens(y), np.roll(X, 3, axis=1))


@pytest.mark.parametrize("form", ["plain", "raised", "direct"])
def test_token_batched_product_on_ciphertexts_decrypts_to_X_times_W(form):
    prm, ctx, sk = _toy_ctx()
    level = 3
    plan = packing.make_plan(ctx.S, 64, 64, tokens=True)           # t = 4 tokens, r_i = 16, r_o = 4
    rng = np.random.default_rng(8)
    X, W = rng.normal(size=(plan.t, 64)) * 0.5, rng.normal(size=(64, 64)) * 0.1
    steps = sorted(set(vmm.direct_giant_steps(plan)) | set(plan.all_steps()))
    keys = ctx.keygen_rotations(sk, steps, 2)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(plan.pack_tokens(X), prm.L), 3), level)
    diags = plan.diagonals(W)
    r0, p0 = ctx.rot_count, ctx.ptmul_count
    if form == "plain":
        y = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, [[ctx.encode(v, level) for v in row] for row in diags])
    else:
        ext = [[ctx.encode_ext(v, level) for v in row] for row in diags]
        fn = vmm.vmm_pt_double_hoisted if form == "raised" else vmm.vmm_pt_direct_giants
        y = fn(ctx, keys, plan, ct, ext)
    assert (plan.r_i, plan.r_o) == (16, 4)
    assert ctx.rot_count - r0 == 18 and ctx.ptmul_count - p0 == 64
    assert y.level == level - 1
    out = ctx.decrypt(sk, y)
    assert np.abs(plan.unpack_tokens(out.real) - X @ W).max() < TOL
    assert np.abs(out.imag).max() < TOL


@pytest.mark.parametrize("r_i", [0, 4])
def test_group_append_builds_the_cache_layouts_and_matches_token_by_token(r_i):
    """Slot level: appending whole groups gives exactly pack_k / pack_v of the plain matrices (the
    definition of the layouts, Sec. 5.1-5.2), and so does appending the same tokens one by one."""
    lay = packing.KvLayout(512, 4, 8, r_i)                          # t = 16
    groups = 3
    ntok = groups * lay.t
    rng = np.random.default_rng(r_i)
    K, V = rng.normal(size=(ntok, 4, 8)), rng.normal(size=(ntok, 4, 8))
    ops = vmm.SlotOps()
    kc, vc = [], [None] * lay.E
    for c in range(groups):
        kg = sum(lay.pack_vec(K[c * lay.t + tau], tau) for tau in range(lay.t))
        vg = sum(lay.pack_vec(V[c * lay.t + tau], tau) for tau in range(lay.t))
        assert np.array_equal(kg, lay.pack_k(K[:(c + 1) * lay.t], c))      # a group IS a K ciphertext
        r0, p0 = ops.rotations, ops.pt_mults
        vmm.kv_append_group(ops, lay, kc, vc, c, kg, vg, np.ones(lay.S),
                            [lay.v_append_group_mask(k, c) for k in range(lay.E)])
        assert (ops.rotations - r0, ops.pt_mults - p0) == (lay.r_o - 1, lay.E + 1)
    for c in range(groups):
        assert np.array_equal(kc[c], lay.pack_k(K, c))
    for k in range(lay.E):
        assert np.array_equal(vc[k], lay.pack_v(V, k))
    k1, v1 = [], [None] * lay.E
    for n in range(ntok):
        tau = n % lay.t
        vmm.kv_append(vmm.SlotOps(), lay, k1, v1, n, lay.pack_vec(K[n], tau), lay.pack_vec(V[n], tau),
                      lay.residue_mask(tau), [lay.v_append_mask(k, n) for k in range(lay.E)])
    assert all(np.array_equal(a, b) for a, b in zip(kc, k1))
    assert all(np.array_equal(a, b) for a, b in zip(vc, v1))
    # the masks of one group tile the whole ciphertext: every slot is taken by exactly one V ciphertext
    # (before the stored rotation), because block row e of group c goes to V ciphertext (c - e) mod E
    tot = sum(np.roll(lay.v_append_group_mask(k, 1), -lay.v_shift(k)) for k in range(lay.E))
    assert np.array_equal(tot, np.ones(lay.S))


def test_group_rope_turns_every_residue_by_its_own_token():
    lay = packing.KvLayout(512, 4, 8)          # t = 16
    c = 5
    rng = np.random.default_rng(4)
    vs = rng.normal(size=(lay.t, 4, 8))
    slots = sum(lay.pack_vec(vs[tau], tau) for tau in range(lay.t))
    ops = vmm.SlotOps()
    out = vmm.rope(ops, lay, slots, lay.rope_plaintexts_group(c))
    assert (ops.rotations, ops.pt_mults) == (2, 3)
    for tau in range(lay.t):
        assert np.abs(lay.unpack_vec(out, tau) - _rope_reference(vs[tau], c * lay.t + tau)).max() < 1e-12


# ---- the whole product in the extended basis: ladders unrolled into hoisted rotations -----------------
@pytest.mark.parametrize("steps", [[], [3], [7, 14], [7, 14, 28], [1, -2, 4, -8], [5, 10, 20, 40, 80, 160, 320]])
def test_ladder_groups_reproduce_the_rotate_and_add_ladder_on_slots(steps):
    rng = np.random.default_rng(len(steps))
    v = rng.normal(size=1024)
    want = v.copy()
    for s in steps:
        want = want + np.roll(want, -s)
    got = v.copy()
    groups = vmm.ladder_groups(steps)
    for amounts in groups:
        assert 1 <= len(amounts) <= 7 and len(set(a % 1024 for a in amounts)) == len(amounts)
        got = got + sum(np.roll(got, -a) for a in amounts)
    assert np.abs(got - want).max() < 1e-9
    assert len(groups) == (len(steps) + 2) // 3
    sizes = [len(g).bit_length() for g in groups]                  # 2^g - 1 amounts -> g steps
    assert sum(sizes) == len(steps) and (not sizes or max(sizes) - min(sizes) <= 1) and sizes == sorted(sizes, reverse=True)


def test_rotsum_raised_against_separate_rotations():
    """One amount from a freshly raised ciphertext: exact (ModDown(u + P a) = ModDown(u) + a).
    Several amounts from a sum with full special limbs: the message of x + sum_a Rot(x, a)."""
    prm, ctx, sk = _toy_ctx()
    keys = ctx.keygen_rotations(sk, [3, 5, 8], 2)
    rng = np.random.default_rng(5)
    z, w = rng.normal(size=(2, ctx.S))
    level = 3
    x = ctx.level_drop(ctx.encrypt(sk, ctx.encode(z, prm.L), 3), level)
    got = ctx.moddown_ct(ctx.rotsum_raised(ctx.raise_ct(x), level, [5], keys), level, x.scale)
    want = ctx.ct_add(x, ctx.rotate_hoisted(x, ctx.hoist(x), 5, keys))
    assert all(np.array_equal(a, b) for a, b in zip(got.c, want.c))
    r0 = ctx.rot_count
    R = ctx.rotsum_raised(ctx.raise_ct(x), level, [3, 5, 8], keys)       # special limbs now full
    assert ctx.rot_count - r0 == 3 and R[0][level + 1:].any()
    R2 = ctx.rotsum_raised(R, level, [3, 8], keys)
    m = ctx.decrypt(sk, ctx.moddown_ct(R2, level, x.scale)).real
    s1 = z + np.roll(z, -3) + np.roll(z, -5) + np.roll(z, -8)
    assert np.abs(m - (s1 + np.roll(s1, -3) + np.roll(s1, -8))).max() < 1e-6


@pytest.mark.parametrize("d_in,d_out,level,tau", [(64, 64, 3, 0), (16, 64, 2, 0), (64, 16, 4, 0), (32, 32, 1, 3),
                                                  (16, 16, 3, 9), (256, 256, 2, 0)])
def test_unrolled_vmm_decrypts_to_x_times_W(d_in, d_out, level, tau):
    """(16, 16) on 256 slots has four-step ladders (two runs of two); (256, 256) has none."""
    prm, ctx, sk = _toy_ctx()
    x, W = inputs.vmm_inputs(7, d_in, d_out, "normal", 0.1)
    plan = packing.make_plan(ctx.S, d_in, d_out, tau=tau)
    steps = vmm.unrolled_steps(plan)
    npre, nred = len(plan.pre_steps), len(plan.reduce_steps)
    ladder = lambda L: sum(len(g) for g in vmm.ladder_groups(list(range(L))))
    assert len(steps) == ladder(npre) + plan.r_i - 1 + plan.r_o - 1 + ladder(nred)
    keys = ctx.keygen_rotations(sk, sorted(set(steps) | set(vmm.direct_giant_steps(plan))), 2)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3), level)
    ext = [[ctx.encode_ext(v, level) for v in row] for row in plan.diagonals(W)]
    r0, p0 = ctx.rot_count, ctx.ptmul_count
    y = vmm.vmm_pt_unrolled(ctx, keys, plan, ct, ext)
    assert ctx.rot_count - r0 == len(steps) and ctx.ptmul_count - p0 == plan.r_i * plan.r_o
    assert y.level == level - 1
    assert np.abs(plan.unpack_output(ctx.decrypt(sk, y).real) - x @ W).max() < TOL
    other = vmm.vmm_pt_direct_giants(ctx, keys, plan, ct, ext)
    assert abs(y.scale / other.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, y) - ctx.decrypt(sk, other)).max() < 1e-6
    if npre == 0 and nred == 0:
        # nothing to unroll: the same computation, bit for bit
        assert np.array_equal(ctx.canonical(y), ctx.canonical(other))


def test_unrolled_qk_scores_decrypt_to_q_times_K_transposed():
    """The sum over the E dims in the extended basis: same scores as the ladder form (and as the
    float64 product); for E = 8 one run of three steps, seven hoisted rotations per key ciphertext
    instead of three dependent ones; for E = 16 two runs of two."""
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    sk = ctx.keygen_secret(1)
    for H, E in ((4, 8), (2, 16)):
        lay = packing.KvLayout(ctx.S, H, E)             # t = 8
        ntok = 2 * lay.t + 3
        q, K, V, s = inputs.attention_inputs(4, H, 2, E, ntok)
        steps = vmm.qk_unrolled_steps(lay)
        if E == 8:
            assert steps == [-1, -2, -4, 32, 64, 96, 128, 160, 192, 224]
        else:
            assert steps == [-1, -2, -4, 16, 32, 48, 64, 128, 192]
        keys = ctx.keygen_rotations(sk, sorted(set(steps) | set(lay.qk_steps())), 2, with_relin=True)
        enc = lambda v, lv, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), lv)
        kc = [enc(lay.pack_k(K, c), L - 1, 100 + c) for c in range(3)]
        cq = enc(lay.pack_vec(q), L - 1, 10)
        masks = [ctx.encode(lay.qk_mask(c), L - 2) for c in range(3)]
        r0 = ctx.rot_count
        m = vmm.qk_scores_unrolled(ctx, keys, lay, cq, kc, masks)
        assert ctx.rot_count - r0 == 3 + 3 * (len(steps) - 3)
        assert m.level == L - 3
        got = lay.unpack_scores(ctx.decrypt(sk, m).real, ntok)
        assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
        ladder = vmm.qk_scores(vmm.CkksOps(ctx, keys), lay, cq, kc, masks)
        assert abs(m.scale / ladder.scale - 1) < 1e-12
        assert np.abs(ctx.decrypt(sk, m) - ctx.decrypt(sk, ladder)).max() < 1e-6


def test_inner_rotations_let_a_query_group_meet_every_key_residue():
    """Sec. 5.4 on slots: t queries in one vector (token tau at residue tau); for every delta the
    inner rotation followed by the un-replicated q K^T gives, at (c, h, tau'), the score of query
    (tau' - delta) mod t against key token c t + tau'; over all delta every pair appears once."""
    lay = packing.KvLayout(256, 4, 8)                   # t = 8
    rng = np.random.default_rng(6)
    Q = rng.normal(size=(lay.t, 4, 8))
    K = rng.normal(size=(2 * lay.t, 4, 8))
    qg = sum(lay.pack_vec(Q[tau], tau) for tau in range(lay.t))
    kc = [lay.pack_k(K, c) for c in range(2)]
    masks = [lay.qk_mask(c) for c in range(2)]
    full = np.einsum("ahe,nhe->ahn", Q, K)              # [query, head, key]
    seen = np.zeros((lay.t, 2 * lay.t), dtype=int)
    for delta in range(lay.t):
        ops = vmm.SlotOps()
        x = qg if delta == 0 else vmm.inner_rotate(ops, lay, qg, delta, lay.inner_rotation_plaintexts(delta))
        if delta:
            assert (ops.rotations, ops.pt_mults) == (2, 3)
            want = np.zeros(lay.S)
            for tau in range(lay.t):
                want += lay.pack_vec(Q[tau], (tau + delta) % lay.t)
            assert np.array_equal(x, want)
        r0 = ops.rotations
        sc = vmm.qk_scores(ops, lay, x, kc, masks, replicate=False)
        assert ops.rotations - r0 == 2 * 3              # only the sums over the 8 dims
        got = lay.unpack_scores(sc, 2 * lay.t)          # [head, key]
        for n in range(2 * lay.t):
            a = (n % lay.t - delta) % lay.t
            assert np.abs(got[:, n] - full[a, :, n]).max() < 1e-12
            seen[a, n] += 1
    assert np.array_equal(seen, np.ones_like(seen))


@pytest.mark.parametrize("r_i", [0, 4])
def test_unrolled_scores_times_v_decrypts_to_s_times_V(r_i):
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    lay = packing.KvLayout(ctx.S, 4, 8, r_i)             # t = 8
    ntok = 3 * lay.t - 1
    q, K, V, s = inputs.attention_inputs(5, 4, 2, 8, ntok)
    sk = ctx.keygen_secret(1)
    steps = vmm.sv_unrolled_steps(lay)
    assert len(steps) == (lay.r_i - 1) + (lay.r_o - 1) + 7
    keys = ctx.keygen_rotations(sk, sorted(set(steps) | set(lay.sv_steps())), 2, with_relin=True)
    enc = lambda v, lv, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), lv)
    vc = [enc(lay.pack_v(V, k), L - 1, 300 + k) for k in range(lay.E)]
    cs = enc(lay.pack_scores(s), L - 1, 50)
    r0 = ctx.rot_count
    a = vmm.score_times_v_unrolled(ctx, keys, lay, cs, vc)
    assert ctx.rot_count - r0 == len(steps) and a.level == L - 2
    assert np.abs(lay.unpack_vec(ctx.decrypt(sk, a).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL
    ladder = vmm.score_times_v(vmm.CkksOps(ctx, keys), lay, cs, vc)
    assert abs(a.scale / ladder.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, a) - ctx.decrypt(sk, ladder)).max() < 1e-6


@pytest.mark.parametrize("r_i", [0, 2])
def test_group_attention_on_slots_is_Q_K_transposed_times_V_for_every_query(r_i):
    """Sec. 5.4 end to end on slots: for every delta the query group is inner-rotated, meets the keys
    (un-replicated q K^T), the scores meet V WITHOUT the sum over the residues, and the partial result
    (at the key's residue) is inner-rotated back by t - delta to the query's residue; the sum over
    delta is, for each of the t queries, the plain product of its scores with V."""
    lay = packing.KvLayout(256, 4, 8, r_i)              # t = 8
    rng = np.random.default_rng(16)
    nk = 3
    Q = rng.normal(size=(lay.t, 4, 8))
    K = rng.normal(size=(nk * lay.t, 4, 8))
    V = rng.normal(size=(nk * lay.t, 4, 8))
    qg = sum(lay.pack_vec(Q[tau], tau) for tau in range(lay.t))
    kc = [lay.pack_k(K, c) for c in range(nk)]
    vc = [lay.pack_v(V, k) for k in range(lay.E)]
    masks = [lay.qk_mask(c) for c in range(nk)]
    ops = vmm.SlotOps()
    out = np.zeros(lay.S)
    for delta in range(lay.t):
        x = qg if delta == 0 else vmm.inner_rotate(ops, lay, qg, delta, lay.inner_rotation_plaintexts(delta))
        sc = vmm.qk_scores(ops, lay, x, kc, masks, replicate=False)
        r0 = ops.rotations
        part = vmm.score_times_v(ops, lay, sc, vc, reduce=False)
        assert ops.rotations - r0 == lay.r_i - 1 + lay.r_o - 1
        # a partial result by hand: keys of residue tau' only, query (tau' - delta) mod t
        for tau in (0, 5):
            a = (tau - delta) % lay.t
            want = sum(np.einsum("he,he->h", Q[a], K[c * lay.t + tau])[:, None] * V[c * lay.t + tau] for c in range(nk))
            assert np.abs(lay.unpack_vec(part, tau) - want).max() < 1e-9
        back = (lay.t - delta) % lay.t
        out = out + (part if back == 0 else vmm.inner_rotate(ops, lay, part, back, lay.inner_rotation_plaintexts(back)))
    att = np.einsum("ahn,nhe->ahe", np.einsum("ahe,nhe->ahn", Q, K), V)
    for tau in range(lay.t):
        assert np.abs(lay.unpack_vec(out, tau) - att[tau]).max() < 1e-9


def test_group_scores_times_v_on_ciphertexts_in_both_forms():
    """reduce=False on ciphertexts: the ladder form and the extended-basis form decrypt to the
    per-residue sums, at the level and scale of the reduced call."""
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    lay = packing.KvLayout(ctx.S, 4, 8, 4)               # t = 8
    ntok = 3 * lay.t
    q, K, V, s = inputs.attention_inputs(7, 4, 2, 8, ntok)
    sk = ctx.keygen_secret(1)
    steps = [a for a in vmm.sv_unrolled_steps(lay) if a % lay.t == 0]
    assert len(steps) == (lay.r_i - 1) + (lay.r_o - 1)
    keys = ctx.keygen_rotations(sk, sorted(set(steps) | {a for a in lay.sv_steps() if a % lay.t == 0}), 2, with_relin=True)
    enc = lambda v, lv, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), lv)
    vc = [enc(lay.pack_v(V, k), L - 1, 300 + k) for k in range(lay.E)]
    cs = enc(lay.pack_scores(s), L - 1, 50)
    r0 = ctx.rot_count
    a = vmm.score_times_v_unrolled(ctx, keys, lay, cs, vc, reduce=False)
    assert ctx.rot_count - r0 == len(steps) and a.level == L - 2
    b = vmm.score_times_v(vmm.CkksOps(ctx, keys), lay, cs, vc, reduce=False)
    assert b.level == L - 2 and abs(a.scale / b.scale - 1) < 1e-12
    da, db = ctx.decrypt(sk, a).real, ctx.decrypt(sk, b).real
    for tau in range(lay.t):
        want = sum(s[:, c * lay.t + tau][:, None] * V[c * lay.t + tau] for c in range(ntok // lay.t))
        assert np.abs(lay.unpack_vec(da, tau) - want).max() < TOL
        assert np.abs(lay.unpack_vec(db, tau) - want).max() < TOL


@pytest.mark.parametrize("shared", [1, 2, 8])
def test_mask_before_the_shared_rotations_gives_the_same_scores_on_slots(shared):
    """The mask moved inside the last `shared` terms of the sum over the dims: identical slot vector
    (not only the kept copy), shared - 1 rotations for the whole cache plus log2(E / shared) per key
    ciphertext."""
    lay = packing.KvLayout(256, 4, 8)                   # t = 8, E = 8
    nk = 5
    ntok = nk * lay.t - 3
    q, K, V, s = inputs.attention_inputs(9, 4, 2, 8, ntok)
    kc = [lay.pack_k(K, c) for c in range(nk)]
    ops, ops2 = vmm.SlotOps(), vmm.SlotOps()
    ref = vmm.qk_scores(ops, lay, lay.pack_vec(q), kc, [lay.qk_mask(c) for c in range(nk)])
    got = vmm.qk_scores_shared_ops(ops2, lay, lay.pack_vec(q), kc, [lay.qk_mask(b) for b in range(lay.E)], shared)
    assert np.abs(got - ref).max() < 1e-12
    assert np.abs(lay.unpack_scores(got, ntok) - np.einsum("he,nhe->hn", q, K)).max() < 1e-12
    log2 = lambda x: x.bit_length() - 1
    assert ops2.rotations == 3 + nk * log2(lay.E // shared) + shared - 1
    assert ops2.pt_mults == nk * shared
    assert len(vmm.qk_shared_steps(lay, shared)) >= 3 + shared - 1


@pytest.mark.parametrize("shared", [2, 8])
def test_shared_dim_rotations_on_ciphertexts_decrypt_to_q_times_K_transposed(shared):
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    sk = ctx.keygen_secret(1)
    lay = packing.KvLayout(ctx.S, 4, 8)                 # t = 8
    ntok = 3 * lay.t - 2
    q, K, V, s = inputs.attention_inputs(4, 4, 2, 8, ntok)
    steps = vmm.qk_shared_steps(lay, shared)
    keys = ctx.keygen_rotations(sk, sorted(set(steps) | set(lay.qk_steps())), 2, with_relin=True)
    enc = lambda v, lv, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), lv)
    kc = [enc(lay.pack_k(K, c), L - 1, 100 + c) for c in range(3)]
    cq = enc(lay.pack_vec(q), L - 1, 10)
    masks = [ctx.encode(lay.qk_mask(b), L - 2) for b in range(lay.E)]
    r0 = ctx.rot_count
    m = vmm.qk_scores_shared(ctx, keys, lay, cq, kc, masks, shared)
    assert ctx.rot_count - r0 == len(steps) + 2 * (len(steps) - 3 - (shared - 1))    # the per-ciphertext part three times
    assert m.level == L - 3
    got = lay.unpack_scores(ctx.decrypt(sk, m).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    ladder = vmm.qk_scores(vmm.CkksOps(ctx, keys), lay, cq, kc, masks[:3])
    assert abs(m.scale / ladder.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, m) - ctx.decrypt(sk, ladder)).max() < 1e-6
    generic = vmm.qk_scores_shared_ops(vmm.CkksOps(ctx, keys), lay, cq, kc, masks, shared)
    assert np.abs(ctx.decrypt(sk, m) - ctx.decrypt(sk, generic)).max() < 1e-6


@pytest.mark.parametrize("r_i", [0, 2, 4])
def test_key_index_gives_the_scores_of_the_printed_order_on_slots(r_i):
    """The key index (copy c of D_k = dim (c + k) of key group c) turns q K^T into a diagonal product: the
    same slot vector as qk_scores (every slot, not only after decoding), no mask, no sum over the dims per
    key ciphertext; and appending token by token, or a group at once, builds exactly pack_k_index."""
    lay = packing.KvLayout(256, 4, 8, r_i)              # t = 8, E = 8
    nk = 5
    ntok = nk * lay.t - 3
    q, K, V, s = inputs.attention_inputs(9, 4, 2, 8, ntok)
    kc = [lay.pack_k(K, c) for c in range(nk)]
    ref = vmm.qk_scores(vmm.SlotOps(), lay, lay.pack_vec(q), kc, [lay.qk_mask(c) for c in range(nk)])
    ops = vmm.SlotOps()
    xc = [lay.pack_k_index(K, k) for k in range(lay.E)]
    got = vmm.qk_scores_indexed(ops, lay, lay.pack_vec(q), xc)
    assert np.abs(got - ref).max() < 1e-12
    assert np.abs(got - lay.pack_scores(np.einsum("he,nhe->hn", q, K))).max() < 1e-12
    assert ops.rotations == 3 + (lay.r_i - 1) + (lay.r_o - 1) and ops.pt_mults == 0
    # a brute-force reading of the layout: ciphertext g r_i + j, copy b = dim (b + j) of key group b - g r_i
    for k in (0, 3, lay.E - 1):
        g, j = k // lay.r_i, k % lay.r_i
        for b in (0, 5):
            for tau in (0, 6):
                n = ((b - g * lay.r_i) % lay.E) * lay.t + tau
                want = K[n, 2, (b + j) % lay.E] if n < ntok else 0.0
                assert xc[k][lay.slot(b, 2, tau)] == want
    # appends: two groups at once, then single tokens
    ops = vmm.SlotOps()
    k_cts, v_cts, x_cts = [], [None] * lay.E, [None] * lay.E
    for c in range(2):
        kg = sum(lay.pack_vec(K[c * lay.t + tau], tau) for tau in range(lay.t)) + 0.0
        vg = sum(lay.pack_vec(V[c * lay.t + tau], tau) for tau in range(lay.t))
        vmm.kv_append_group(ops, lay, k_cts, v_cts, c, kg, vg, np.ones(lay.S),
                            [lay.v_append_group_mask(k, c) for k in range(lay.E)],
                            x_cts, [lay.k_index_append_group_mask(k, c) for k in range(lay.E)])
    for n in range(2 * lay.t, ntok):
        junk = np.roll(lay.pack_vec(K[n] * 7, (n + 1) % lay.t), 0)      # other residues hold partial sums
        vmm.kv_append(ops, lay, k_cts, v_cts, n, lay.pack_vec(K[n], n % lay.t) + junk, lay.pack_vec(V[n], n % lay.t),
                      lay.residue_mask(n % lay.t), [lay.v_append_mask(k, n) for k in range(lay.E)],
                      x_cts, [lay.k_index_append_mask(k, n) for k in range(lay.E)])
    for k in range(lay.E):
        assert np.abs(x_cts[k] - xc[k]).max() < 1e-12
    for c in range(nk):
        assert np.abs(k_cts[c] - kc[c]).max() < 1e-12


@pytest.mark.parametrize("r_i", [0, 4])
def test_key_index_on_ciphertexts_decrypts_to_q_times_K_transposed(r_i):
    prm = params.toy(n=512, n_qi=4, n_p=1, alpha=1)
    ctx = ckks.Context(prm)
    L = prm.L
    sk = ctx.keygen_secret(1)
    lay = packing.KvLayout(ctx.S, 4, 8, r_i)            # t = 8
    ntok = 3 * lay.t - 2
    q, K, V, s = inputs.attention_inputs(4, 4, 2, 8, ntok)
    steps = sorted(set(vmm.sv_unrolled_steps(lay)) | set(lay.sv_steps()) | set(lay.qk_steps()))
    keys = ctx.keygen_rotations(sk, steps, 2, with_relin=True)
    enc = lambda v, lv, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), lv)
    xc = [enc(lay.pack_k_index(K, k), L - 1, 100 + k) for k in range(lay.E)]
    cq = enc(lay.pack_vec(q), L - 1, 10)
    want = np.einsum("he,nhe->hn", q, K)
    ops = vmm.CkksOps(ctx, keys)
    a = vmm.qk_scores_indexed(ops, lay, cq, xc)
    assert a.level == L - 2                              # one level, not two
    assert np.abs(lay.unpack_scores(ctx.decrypt(sk, a).real, ntok) - want).max() < TOL
    b = vmm.qk_scores_indexed(ops, lay, cq, xc,
                              sv=lambda c, x: vmm.score_times_v_unrolled(ctx, keys, lay, c, x, reduce=False))
    assert b.level == L - 2 and abs(a.scale / b.scale - 1) < 1e-12
    assert np.abs(ctx.decrypt(sk, a) - ctx.decrypt(sk, b)).max() < 1e-6


# ---- grouped-query attention against a cache that stores every KV head once ---------------------------------
def _gqa_inputs(seed, H, Hkv, E, ntok):
    rng = np.random.default_rng(seed)
    q = rng.normal(size=(H, E))
    K, V = rng.normal(size=(ntok, Hkv, E)), rng.normal(size=(ntok, Hkv, E))
    s = rng.uniform(0, 1, size=(H, ntok))
    return q, K, V, s / s.sum(axis=1, keepdims=True)


@pytest.mark.parametrize("S,H,Hkv,E,r_i,ntok", [(2048, 8, 2, 16, 4, 150), (2048, 4, 2, 32, 0, 37), (512, 8, 1, 8, 2, 64)])
def test_gqa_layout_on_slots_is_grouped_attention_and_matches_the_replicated_layout(S, H, Hkv, E, r_i, ntok):
    """Slot level (no cryptography): the query layout and the cache layout meet slot for slot; q K^T and scores V
    through the G passes equal the einsum with each KV head shared by G query heads, and equal, number for
    number, what the paper's layout gives with every KV head repeated G times; the cache is 1/G as many
    ciphertexts, the ciphertext products as many as before."""
    glay = packing.GqaLayout(S, H, Hkv, E, r_i)
    G, t, kvl = glay.G, glay.t, glay.kv
    for e, hk, g, tau in ((0, 0, 0, 0), (E - 1, Hkv - 1, G - 1, t - 1), (3, Hkv - 1, 1, t // 2)):
        assert glay.q.slot(e, hk * G + g, tau) == kvl.slot(e, hk, g * t + tau)
    q, K, V, s = _gqa_inputs(S + H, H, Hkv, E, ntok)
    Krep, Vrep = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)
    nk = -(-ntok // kvl.t)
    k_cts = [kvl.pack_k(K, c) for c in range(nk)]
    v_cts = [kvl.pack_v(V, k) for k in range(E)]
    rots = {d: kvl.inner_rotation_plaintexts(glay.inner_delta(d)) for d in range(1, G)}
    ops = vmm.SlotOps()
    outs = vmm.gqa_qk_scores(ops, glay, glay.q.pack_vec(q), k_cts, [kvl.qk_mask(c) for c in range(nk)], rots)
    assert len(outs) == G and ops.ct_mults == G * nk
    m = glay.unpack_scores(outs, ntok)
    want = np.einsum("he,nhe->hn", q, Krep)
    assert np.abs(m - want).max() < 1e-10
    # every slot of every pass is either a score or zero: nothing is computed twice
    assert sum(int(np.count_nonzero(np.abs(o) > 1e-300)) for o in outs) <= H * nk * kvl.t
    # the paper's layout with repeated heads: the same numbers from G times as many key ciphertexts
    rep = packing.KvLayout(S, H, E, r_i)
    nk_rep = -(-ntok // rep.t)
    ops_r = vmm.SlotOps()
    m_rep = vmm.qk_scores(ops_r, rep, rep.pack_vec(q), [rep.pack_k(Krep, c) for c in range(nk_rep)],
                          [rep.qk_mask(c) for c in range(nk_rep)])
    assert np.abs(rep.unpack_scores(m_rep, ntok) - m).max() < 1e-10
    assert G * (nk - 1) < nk_rep <= G * nk and ops_r.ct_mults == nk_rep
    # scores V
    ops = vmm.SlotOps()
    att = vmm.gqa_score_times_v(ops, glay, glay.pack_scores(s), v_cts, rots)
    assert ops.ct_mults == G * E
    want_att = np.einsum("hn,nhe->he", s, Vrep)
    assert np.abs(glay.q.unpack_vec(att) - want_att).max() < 1e-10
    att_rep = vmm.score_times_v(vmm.SlotOps(), rep, rep.pack_scores(s), [rep.pack_v(Vrep, k) for k in range(E)])
    assert np.abs(rep.unpack_vec(att_rep) - glay.q.unpack_vec(att)).max() < 1e-10
    # pack_scores / unpack_scores are inverse to each other and cover every (head, token) once
    assert np.array_equal(glay.unpack_scores(glay.pack_scores(s), ntok), s)
    assert sum(int(np.count_nonzero(v)) for v in glay.pack_scores(s)) == H * ntok


def test_gqa_attention_on_ciphertexts_decrypts_to_grouped_attention():
    """The same two products on oracle ciphertexts (config-1 ring: 8 query heads on 2 KV heads, 16 dims):
    decrypted scores and outputs within 1e-4 of float64, levels as documented."""
    prm = params.config1()
    ctx = ckks.Context(prm)
    H, Hkv, E, ntok = 8, 2, 16, 70
    glay = packing.GqaLayout(ctx.S, H, Hkv, E, 4)
    kvl, G, L = glay.kv, glay.G, prm.L
    q, K, V, s = _gqa_inputs(5, H, Hkv, E, ntok)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, glay.qk_steps() + glay.sv_steps(), 2, with_relin=True)
    lv = L - 1
    enc = lambda v, level, seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(v, L), seed), level)
    nk = -(-ntok // kvl.t)
    k_cts = [enc(kvl.pack_k(K, c), lv, 100 + c) for c in range(nk)]
    v_cts = [enc(kvl.pack_v(V, k), lv, 300 + k) for k in range(E)]
    ops = vmm.CkksOps(ctx, keys)

    def rot_pts(level):
        ql = float(ctx.mod[level])
        return {d: [ctx.encode(p, level, ql) for p in kvl.inner_rotation_plaintexts(glay.inner_delta(d))] for d in range(1, G)}
    masks = [ctx.encode(kvl.qk_mask(c), lv - 1, float(ctx.mod[lv - 1])) for c in range(nk)]
    outs = vmm.gqa_qk_scores(ops, glay, enc(glay.q.pack_vec(q), lv + 1, 10), k_cts, masks, rot_pts(lv + 1))
    assert all(o.level == lv - 2 for o in outs)
    m = glay.unpack_scores([ctx.decrypt(sk, o).real for o in outs], ntok)
    assert np.abs(m - np.einsum("he,nhe->hn", q, np.repeat(K, G, axis=1))).max() < 1e-4
    cs = [enc(v, lv, 50 + d) for d, v in enumerate(glay.pack_scores(s))]
    att = vmm.gqa_score_times_v(ops, glay, cs, v_cts, rot_pts(lv - 1))
    assert att.level == lv - 2
    got = glay.q.unpack_vec(ctx.decrypt(sk, att).real)
    assert np.abs(got - np.einsum("hn,nhe->he", s, np.repeat(V, G, axis=1))).max() < 1e-4


def test_twelve_heads_are_padded_to_sixteen_and_attention_is_unchanged():
    """GPT2-base (Table 3: 12 heads of 64 dims, width 768): the layout pads the head count to the next power of
    two the way Table 4 pads the width to 1024 (= 16 x 64).  On slots q K^T and scores V are the einsum over the
    12 real heads; the padding heads' slots stay zero."""
    S, H, E, ntok = 32768, 12, 64, 75
    lay = packing.KvLayout(S, H, E, 8)
    assert (lay.heads, lay.H, lay.H * lay.E, lay.t, lay.capacity) == (12, 16, 1024, 32, 2048)
    rng = np.random.default_rng(12)
    q = rng.normal(size=(H, E))
    K, V = rng.normal(size=(ntok, H, E)), rng.normal(size=(ntok, H, E))
    s = rng.uniform(0, 1, size=(H, ntok))
    nk = -(-ntok // lay.t)
    ops = vmm.SlotOps()
    m = vmm.qk_scores(ops, lay, lay.pack_vec(q), [lay.pack_k(K, c) for c in range(nk)], [lay.qk_mask(c) for c in range(nk)])
    assert np.abs(lay.unpack_scores(m, ntok) - np.einsum("he,nhe->hn", q, K)).max() < 1e-10
    pad = [lay.slot(c, h, tau) for c in range(E) for h in range(12, 16) for tau in range(lay.t)]
    assert not np.any(m[pad])
    att = vmm.score_times_v(ops, lay, lay.pack_scores(s), [lay.pack_v(V, k) for k in range(E)])
    assert np.abs(lay.unpack_vec(att) - np.einsum("hn,nhe->he", s, V)).max() < 1e-10
    assert not np.any(att[[lay.slot(e, h, 0) for e in range(E) for h in range(12, 16)]])
    # the packed product that feeds it: the padded width 1024 takes the 20 rotations of Table 4
    assert packing.make_plan(S, 1024, 1024).n_rotations == 20
