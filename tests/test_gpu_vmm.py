"""GPU parity of the packed products: vmm_pt (Algorithm 1) and vmm_kv (Sec. 5) against the
oracle, limbs bit for bit, and against the float64 products within 1e-4."""
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


def _enc_both(e, slots, level, seed, scale=None):
    octx, gctx = e["octx"], e["gctx"]
    scale = octx.prm.scale if scale is None else scale
    coeffs = octx.encode_coeffs(slots, scale)
    top = octx.prm.L
    o = octx.level_drop(octx.encrypt(e["osk"], octx.pt_from_coeffs(coeffs, top, scale), seed), level)
    g = gctx.encrypt(e["gsk"], gctx.pt_from_coeffs(coeffs, top, scale), seed)
    if level != top:
        g = gctx.level_drop(g, level)
    return o, g


def _same(e, o, g):
    assert g.level == o.level and abs(g.scale / o.scale - 1) < 1e-12
    assert np.array_equal(e["gctx"].ct_export(g), e["octx"].canonical(o))


@pytest.mark.parametrize("d_in,d_out,level,r_i,tau,seed", [
    (64, 64, 4, 0, 0, 0),          # benchmark configuration 1
    (64, 64, 2, 1, 0, 1),          # no baby steps
    (256, 256, 3, 0, 0, 2),        # 32 diagonals: 8 baby x 4 giant steps
    (128, 512, 4, 0, 0, 3),        # expanding
    (512, 128, 2, 0, 0, 4),        # contracting
    (128, 128, 4, 0, 5, 5),        # output on residue 5 (cache append)
])
def test_vmm_pt_matches_oracle_and_float64(env, d_in, d_out, level, r_i, tau, seed):
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    e = env
    octx, gctx = e["octx"], e["gctx"]
    x, W = inputs.vmm_inputs(seed, d_in, d_out, "uniform", 0.05)
    plan = packing.make_plan(octx.S, d_in, d_out, r_i or None, tau)
    scale = octx.prm.scale
    diag_coeffs = [[octx.encode_coeffs(v, scale) for v in row] for row in plan.diagonals(W)]
    odiags = [[octx.pt_from_coeffs(c, level, scale) for c in row] for row in diag_coeffs]
    flat = np.stack([c for row in diag_coeffs for c in row])
    gplan = gctx.vmm_plan(d_in, d_out, level=level, r_i=plan.r_i, tau=tau, coeffs=flat)
    assert (gplan.r_i, gplan.r_o, gplan.n_rotations) == (plan.r_i, plan.r_o, plan.n_rotations)
    assert sorted(set(gplan.steps())) == sorted(set(plan.all_steps()))
    okeys = octx.keygen_rotations(e["osk"], plan.all_steps(), 2)
    gkeys = gctx.keygen_rotations(e["gsk"], gplan.steps(), 2)
    ox, gx = _enc_both(e, plan.pack_input(x), level, 3)
    oy = vmm.vmm_pt(vmm.CkksOps(octx, okeys), plan, ox, odiags)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    _same(e, oy, gy)
    out = gctx.decrypt(e["gsk"], gy)
    assert np.abs(plan.unpack_output(out.real) - x @ W).max() < TOL

    # the library's own diagonal extraction and encoder: within one unit of the oracle's, and
    # the product still decrypts to x W
    gplan2 = gctx.vmm_plan(d_in, d_out, W=W, level=level, r_i=plan.r_i, tau=tau)
    q0 = int(octx.mod[0])
    for j, k in {(0, 0), (plan.r_i - 1, plan.r_o - 1)}:
        got = gplan2.diag_export(j, k)[0].astype(np.int64)
        got = np.where(got > q0 // 2, got - q0, got)
        assert np.abs(got - diag_coeffs[j][k]).max() <= 1
    out2 = gctx.decrypt(e["gsk"], gctx.vmm_pt(gkeys, gplan2, gx))
    assert np.abs(plan.unpack_output(out2.real) - x @ W).max() < TOL


def _raised_case(e, d_in, d_out, level, r_i, tau, seed, direct=False, unrolled=False):
    """vmm_pt with the baby-step sums kept in the extended basis (and, with direct, the giant steps
    unrolled; with unrolled, the two ladders as well) against the oracle's form of it."""
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    octx, gctx = e["octx"], e["gctx"]
    x, W = inputs.vmm_inputs(seed, d_in, d_out, "uniform", 0.05)
    plan = packing.make_plan(octx.S, d_in, d_out, r_i or None, tau)
    scale = octx.prm.scale
    diag_coeffs = [[octx.encode_coeffs(v, scale) for v in row] for row in plan.diagonals(W)]
    odiags = [[octx.pt_from_coeffs_ext(c, level, scale) for c in row] for row in diag_coeffs]
    flat = np.stack([c for row in diag_coeffs for c in row])
    gplan = gctx.vmm_plan(d_in, d_out, level=level, r_i=plan.r_i, tau=tau, coeffs=flat, raised_sums=True,
                          direct_giants=direct, unrolled_ladders=unrolled)
    steps = vmm.unrolled_steps(plan) if unrolled else vmm.direct_giant_steps(plan) if direct else plan.all_steps()
    assert (gplan.r_i, gplan.r_o) == (plan.r_i, plan.r_o)
    assert gplan.n_rotations == (len(steps) if unrolled else plan.n_rotations)
    assert sorted(set(gplan.steps())) == sorted(set(steps)) and (not direct or unrolled or len(gplan.steps()) == plan.n_rotations)
    if unrolled:
        assert gplan.steps() == steps
    # the plaintexts live on level+1+K limbs
    ext = octx.ext_idx(level)
    j, k = plan.r_i - 1, plan.r_o - 1
    assert np.array_equal(gplan.diag_export(j, k), octx.intt(odiags[j][k].m, ext))
    okeys = octx.keygen_rotations(e["osk"], steps, 2)
    gkeys = gctx.keygen_rotations(e["gsk"], gplan.steps(), 2)
    ox, gx = _enc_both(e, plan.pack_input(x), level, 3)
    fn = vmm.vmm_pt_unrolled if unrolled else vmm.vmm_pt_direct_giants if direct else vmm.vmm_pt_double_hoisted
    oy = fn(octx, okeys, plan, ox, odiags)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    _same(e, oy, gy)
    out = gctx.decrypt(e["gsk"], gy)
    assert np.abs(plan.unpack_output(out.real) - x @ W).max() < TOL
    # twice in a row on the same buffers: nothing left over from the first run
    assert np.array_equal(gctx.ct_export(gctx.vmm_pt(gkeys, gplan, gx)), gctx.ct_export(gy))


@pytest.mark.parametrize("d_in,d_out,level,r_i,tau,seed", [
    (64, 64, 4, 0, 0, 0),
    (64, 64, 2, 1, 0, 1),          # no baby steps: only the raised input
    (256, 256, 3, 0, 0, 2),
    (128, 512, 4, 0, 0, 3),
    (512, 128, 1, 0, 0, 4),
    (128, 128, 4, 0, 5, 5),
])
def test_vmm_pt_raised_sums_matches_oracle_and_float64(env, d_in, d_out, level, r_i, tau, seed):
    _raised_case(env, d_in, d_out, level, r_i, tau, seed)


@pytest.mark.parametrize("d_in,d_out,level,r_i,tau,seed", [
    (64, 64, 4, 0, 0, 0),          # one giant step
    (64, 64, 2, 1, 0, 1),          # no baby steps, one giant step
    (512, 512, 3, 4, 0, 2),        # 128 diagonals as 4 baby x 32 giant steps: 31 independent rotations (4 ModDown batches)
    (128, 512, 4, 0, 0, 3),
    (512, 128, 1, 0, 0, 4),
    (128, 128, 4, 2, 5, 5),
])
def test_vmm_pt_direct_giants_matches_oracle_and_float64(env, d_in, d_out, level, r_i, tau, seed):
    _raised_case(env, d_in, d_out, level, r_i, tau, seed, direct=True)


@pytest.mark.parametrize("d_in,d_out,level,r_i,tau,seed", [
    (64, 64, 4, 0, 0, 0),          # t = 32: five-step ladders before and after, runs of three and two
    (64, 64, 2, 1, 0, 1),          # no baby steps
    (512, 512, 3, 4, 0, 2),        # t = 4: two-step ladders; 31 unrolled giant steps
    (128, 512, 4, 0, 0, 3),        # expanding: preprocess ladder of four steps, reduce ladder of two
    (512, 128, 1, 0, 0, 4),        # contracting
    (128, 128, 4, 2, 5, 5),        # output on residue 5: right rotations in the reduce ladder
    (2048, 2048, 3, 0, 0, 6),      # t = 1: no ladders at all
])
def test_vmm_pt_unrolled_ladders_matches_oracle_and_float64(env, d_in, d_out, level, r_i, tau, seed):
    _raised_case(env, d_in, d_out, level, r_i, tau, seed, direct=True, unrolled=True)


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("level", [5, 4, 2])
def test_vmm_pt_raised_sums_with_two_primes_per_digit(level, direct):
    """Digits of two primes and two special primes (level 4: the last digit holds one prime)."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import ckks, params
    from paper_2602_11470_amd import binding as B
    prm = params.toy(n=4096, n_qi=5, n_p=2, alpha=2, hamming=64)
    octx, gctx = ckks.Context(prm), B.Context(4096, 6, 2, 2, 50, 40, 60, 2.0 ** 40, hamming=64)
    try:
        assert gctx.moduli().tolist() == prm.moduli
        e = dict(B=B, octx=octx, gctx=gctx, osk=octx.keygen_secret(1), gsk=gctx.keygen_secret(1), prm=prm)
        _raised_case(e, 128, 128, level, 0, 0, 7, direct)
    finally:
        gctx.close()


@pytest.mark.parametrize("direct", [False, True, "unrolled"])
def test_vmm_pt_replays_from_a_captured_graph(env, direct):
    """cm_vmm_pt only enqueues kernels and device copies on the caller's stream, so it can be
    captured into a HIP graph: every replay (with eager work in between) reproduces the eager
    result bit for bit."""
    import torch
    from paper_2602_11470_amd import inputs
    e = env
    gctx = e["gctx"]
    x, W = inputs.vmm_inputs(9, 256, 256, "uniform", 0.05)
    gplan = gctx.vmm_plan(256, 256, W=W, level=3, raised_sums=bool(direct), direct_giants=bool(direct),
                          unrolled_ladders=direct == "unrolled")
    gkeys = gctx.keygen_rotations(e["gsk"], gplan.steps(), 2)
    slots = np.zeros(gctx.S)
    slots[::gctx.S // 256] = x
    _, gx = _enc_both(e, slots, 3, 4)
    eager = gctx.vmm_pt(gkeys, gplan, gx)                      # also warms the per-level tables
    torch.cuda.synchronize()
    ref = gctx.ct_export(eager).copy()
    out = gctx.vmm_pt(gkeys, gplan, gx)
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        gctx.vmm_pt(gkeys, gplan, gx, out=out)
    for _ in range(3):
        out.buf.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(gctx.ct_export(out), ref)
        gctx.vmm_pt(gkeys, gplan, gx, out=eager)               # eager work between the replays
        torch.cuda.synchronize()
    assert np.abs(gctx.decrypt(e["gsk"], out).real[::gctx.S // 256] - x @ W).max() < TOL


@pytest.mark.parametrize("token,tau,level", [(0, 0, 4), (77, 5, 3), (4095, 2, 1)])
def test_rope_with_fused_extraction_matches_oracle_and_the_textbook_rotation(env, token, tau, level):
    """App. D on 16 heads x 16 dims (t = 8): limbs against the oracle from identical integer
    plaintexts, decrypted result against the rotation of every dim pair, other slots clean."""
    from oracle import packing, vmm
    e = env
    octx, gctx, prm = e["octx"], e["gctx"], e["prm"]
    lay = packing.KvLayout(octx.S, 16, 16)
    rng = np.random.default_rng(token)
    v = rng.normal(size=(16, 16))
    slots = rng.normal(size=octx.S)                      # partial sums everywhere ...
    for h in range(16):
        for d in range(16):
            slots[lay.slot(d, h, tau)] = v[h, d]         # ... except the valid slots
    ox, gx = _enc_both(e, slots, level, 3)
    scale = float(prm.moduli[level])
    coeffs = [octx.encode_coeffs(p, scale) for p in lay.rope_plaintexts(token, tau)]
    grope = gctx.rope(16, 16, level, token, tau, coeffs=np.stack(coeffs))
    assert sorted(grope.steps()) == sorted([lay.rope_step, -lay.rope_step])
    okeys = octx.keygen_rotations(e["osk"], grope.steps(), 2)
    gkeys = gctx.keygen_rotations(e["gsk"], grope.steps(), 2)
    oy = vmm.rope(vmm.CkksOps(octx, okeys), lay, ox, [octx.pt_from_coeffs(c, level, scale) for c in coeffs])
    gy = gctx.rope_apply(gkeys, grope, gx)
    _same(e, oy, gy)
    want = np.empty_like(v)
    for m in range(8):
        th = token * 10000.0 ** (-2.0 * m / 16)
        want[:, 2 * m] = v[:, 2 * m] * np.cos(th) - v[:, 2 * m + 1] * np.sin(th)
        want[:, 2 * m + 1] = v[:, 2 * m + 1] * np.cos(th) + v[:, 2 * m] * np.sin(th)
    # the library's own plaintexts: same message
    gy2 = gctx.rope_apply(gkeys, gctx.rope(16, 16, level, token, tau), gx)
    for g in (gy, gy2):
        out = gctx.decrypt(e["gsk"], g).real
        assert np.abs(lay.unpack_vec(out, tau) - want).max() < TOL
        valid = np.zeros(octx.S, dtype=bool)
        valid[[lay.slot(d, h, tau) for d in range(16) for h in range(16)]] = True
        assert np.abs(out[~valid]).max() < TOL
    with pytest.raises(e["B"].CachemirError) as err:
        gctx.rope_apply(gctx.keygen_rotations(e["gsk"], [lay.rope_step], 2), grope, gx)
    assert err.value.status == -4


@pytest.mark.parametrize("d_in,d_out", [(2048, 2048), (64, 64), (2, 2048), (2048, 2)])
def test_vmm_pt_degenerate_shapes(env, d_in, d_out):
    """d = S (one slot per element: no preprocess and no reduce rotations), the narrowest square
    product the ring allows (d^2 >= S: two diagonals), and the widest expansion / contraction; all
    three forms."""
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    e = env
    octx, gctx = e["octx"], e["gctx"]
    level = 2
    x, W = inputs.vmm_inputs(11, d_in, d_out, "uniform", 0.5 if max(d_in, d_out) < 4 else 0.02)
    plan = packing.make_plan(octx.S, d_in, d_out)
    scale = octx.prm.scale
    diag_coeffs = [[octx.encode_coeffs(v, scale) for v in row] for row in plan.diagonals(W)]
    flat = np.stack([c for row in diag_coeffs for c in row])
    steps = sorted(set(vmm.direct_giant_steps(plan)) | set(plan.all_steps()))
    okeys = octx.keygen_rotations(e["osk"], steps, 2) if steps else {}
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2)
    ox, gx = _enc_both(e, plan.pack_input(x), level, 3)
    for form in ("plain", "raised", "direct"):
        gplan = gctx.vmm_plan(d_in, d_out, level=level, r_i=plan.r_i, coeffs=flat,
                              raised_sums=form != "plain", direct_giants=form == "direct", unrolled_ladders=form == "unrolled")
        assert gplan.n_rotations == plan.n_rotations
        if form == "plain":
            odiags = [[octx.pt_from_coeffs(c, level, scale) for c in row] for row in diag_coeffs]
            oy = vmm.vmm_pt(vmm.CkksOps(octx, okeys), plan, ox, odiags)
        else:
            odiags = [[octx.pt_from_coeffs_ext(c, level, scale) for c in row] for row in diag_coeffs]
            fn = vmm.vmm_pt_direct_giants if form == "direct" else vmm.vmm_pt_double_hoisted
            oy = fn(octx, okeys, plan, ox, odiags)
        gy = gctx.vmm_pt(gkeys, gplan, gx)
        _same(e, oy, gy)
        assert np.abs(plan.unpack_output(gctx.decrypt(e["gsk"], gy).real) - x @ W).max() < TOL


@pytest.mark.parametrize("seed", range(16))
def test_vmm_pt_seeded_sweep_of_shapes_levels_and_forms(env, seed):
    """Shapes, levels, baby-step counts, residues and forms drawn from a seeded generator; every
    case limb for limb against the oracle, and run twice (a race would show as a difference)."""
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    e = env
    octx, gctx = e["octx"], e["gctx"]
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128, 256, 512, 1024]))
    alpha = int(rng.choice([1, 1, 2, 4]))
    shape = rng.choice(["square", "expand", "contract"]) if alpha > 1 and d * alpha <= octx.S else "square"
    d_in, d_out = (d, d) if shape == "square" else (d, d * alpha) if shape == "expand" else (d * alpha, d)
    level = int(rng.integers(1, 5))
    plan0 = packing.make_plan(octx.S, d_in, d_out)
    r_i = int(rng.choice([r for r in (1, 2, 4, 8, 16, 32) if plan0.M % r == 0 and r <= plan0.M]))
    tau = int(rng.integers(0, plan0.t2))
    form = str(rng.choice(["plain", "raised", "direct"]))
    if seed >= 10:
        form = "unrolled"
    plan = packing.make_plan(octx.S, d_in, d_out, r_i, tau)
    x, W = inputs.vmm_inputs(seed, d_in, d_out, "uniform", 0.05)
    scale = octx.prm.scale
    diag_coeffs = [[octx.encode_coeffs(v, scale) for v in row] for row in plan.diagonals(W)]
    flat = np.stack([c for row in diag_coeffs for c in row])
    steps = sorted(set(vmm.unrolled_steps(plan) if form == "unrolled" else
                       vmm.direct_giant_steps(plan) if form == "direct" else plan.all_steps()))
    okeys = octx.keygen_rotations(e["osk"], steps, 2) if steps else {}
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2)
    ox, gx = _enc_both(e, plan.pack_input(x), level, 3)
    gplan = gctx.vmm_plan(d_in, d_out, level=level, r_i=r_i, tau=tau, coeffs=flat,
                          raised_sums=form != "plain", direct_giants=form == "direct", unrolled_ladders=form == "unrolled")
    if form == "plain":
        odiags = [[octx.pt_from_coeffs(c, level, scale) for c in row] for row in diag_coeffs]
        oy = vmm.vmm_pt(vmm.CkksOps(octx, okeys), plan, ox, odiags)
    else:
        odiags = [[octx.pt_from_coeffs_ext(c, level, scale) for c in row] for row in diag_coeffs]
        fn = {"raised": vmm.vmm_pt_double_hoisted, "direct": vmm.vmm_pt_direct_giants, "unrolled": vmm.vmm_pt_unrolled}[form]
        oy = fn(octx, okeys, plan, ox, odiags)
    gy = gctx.vmm_pt(gkeys, gplan, gx)
    _same(e, oy, gy)
    assert np.array_equal(gctx.ct_export(gctx.vmm_pt(gkeys, gplan, gx)), gctx.ct_export(gy))
    assert np.abs(plan.unpack_output(gctx.decrypt(e["gsk"], gy).real) - x @ W).max() < TOL, (d_in, d_out, level, r_i, tau, form)


@pytest.mark.parametrize("direct", [False, True, "unrolled"])
def test_vmm_pt_multi_shares_baby_steps_and_equals_single_products(env, direct):
    """Three projections of one input (different weights, one of them landing on another residue):
    each output of the shared-baby-step call is bit for bit the single product's."""
    from paper_2602_11470_amd import inputs
    e = env
    B, gctx = e["B"], e["gctx"]
    d, level = 256, 3
    x, _ = inputs.vmm_inputs(20, d, d, "uniform", 0.05)
    Ws = [inputs.vmm_inputs(21 + i, d, d, "uniform", 0.05)[1] for i in range(3)]
    plans = [gctx.vmm_plan(d, d, W=W, level=level, tau=(3 if i == 1 else 0), raised_sums=True, direct_giants=bool(direct),
                           unrolled_ladders=direct == "unrolled") for i, W in enumerate(Ws)]
    steps = sorted(set(sum((p.steps() for p in plans), [])))
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2)
    slots = np.zeros(gctx.S)
    t = gctx.S // d
    slots[::t] = x
    _, gx = _enc_both(e, slots, level, 4)
    singles = [gctx.ct_export(gctx.vmm_pt(gkeys, p, gx)).copy() for p in plans]
    outs = gctx.vmm_pt_multi(gkeys, plans, gx)
    for i, (o, ref) in enumerate(zip(outs, singles)):
        assert np.array_equal(gctx.ct_export(o), ref)
        tau = 3 if i == 1 else 0
        assert np.abs(gctx.decrypt(e["gsk"], o).real[tau::t] - x @ Ws[i]).max() < TOL
    plain = gctx.vmm_plan(d, d, W=Ws[0], level=level)
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_pt_multi(gkeys, [plans[0], plain], gx)           # needs the raised form
    assert err.value.status == -1
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_pt_multi(gkeys, [plans[0], plans[0]], gx)        # one work area per plan
    assert err.value.status == -1
    other = gctx.vmm_plan(d, d, W=Ws[0], level=level, r_i=4, raised_sums=True)
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_pt_multi(gkeys, [plans[0], other], gx)           # different baby steps
    assert err.value.status in (-5, -4)


def test_kv_single_token_and_full_cache(env):
    """One token in the cache (a ragged first key ciphertext), then the cache filled to its
    capacity E t: scores and weighted values against float64, and one append too many refused."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx, L = e["B"], e["octx"], e["gctx"], e["prm"].L
    H, E = 64, 4                                             # t = 8, capacity 32 tokens
    lay = packing.KvLayout(octx.S, H, E)
    q, K, V, s = inputs.attention_inputs(6, H, H, E, lay.capacity)
    kv = gctx.kv_create(H, E, L - 1)
    gkeys = gctx.keygen_rotations(e["gsk"], kv.steps(), 2, with_relin=True)
    enc = lambda slots, level, seed: _enc_both(e, slots, level, seed)[1]
    for n in range(lay.capacity):
        tau = n % lay.t
        kv.append(gkeys, enc(lay.pack_vec(K[n], tau), L, 100 + n), enc(lay.pack_vec(V[n], tau), L, 200 + n))
        if n in (0, lay.capacity - 1):
            ntok = n + 1
            gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, enc(lay.pack_vec(q), L - 1, 7))
            got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
            assert np.abs(got - np.einsum("he,nhe->hn", q, K[:ntok])).max() < TOL
            sn = s[:, :ntok] / s[:, :ntok].sum(axis=1, keepdims=True)
            ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, enc(lay.pack_scores(sn), L - 1, 8))
            assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", sn, V[:ntok])).max() < TOL
    with pytest.raises(B.CachemirError) as err:
        kv.append(gkeys, enc(lay.pack_vec(K[0], 0), L, 1), enc(lay.pack_vec(V[0], 0), L, 2))
    assert err.value.status == -5
    empty = gctx.kv_create(H, E, L - 1)
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_kv(gkeys, empty, B.CM_QK, enc(lay.pack_vec(q), L - 1, 7))
    assert err.value.status == -5


def test_vmm_pt_missing_key_and_level_errors(env):
    e = env
    B, gctx = e["B"], e["gctx"]
    W = np.zeros((64, 64))
    gplan = gctx.vmm_plan(64, 64, W=W, level=3)
    gkeys = gctx.keygen_rotations(e["gsk"], gplan.steps()[:-1], 2)
    _, gx = _enc_both(e, np.zeros(8), 3, 1)
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_pt(gkeys, gplan, gx)
    assert err.value.status == -4
    _, gx2 = _enc_both(e, np.zeros(8), 2, 1)
    full = gctx.keygen_rotations(e["gsk"], gplan.steps(), 2)
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_pt(full, gplan, gx2)
    assert err.value.status == -2
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_plan(96, 96, W=np.zeros((96, 96)), level=3)       # not a power of two
    assert err.value.status == -5
    with pytest.raises(B.CachemirError) as err:
        gctx.vmm_plan(32, 32, W=np.zeros((32, 32)), level=3)       # d^2 < S: less than one diagonal
    assert err.value.status == -5
    h, w = B._vp(), np.zeros((64, 64))
    status = B.lib.cm_vmm_plan_create_ex(gctx.h, 64, 64, 0, 0, 3, 0.0, w.ctypes.data, None, 1 << 10, B.C.byref(h))
    assert status == -1 and not h.value                            # unknown flag bit
    status = B.lib.cm_vmm_plan_create_ex(gctx.h, 64, 64, 0, 0, 3, 0.0, None, None, 0, B.C.byref(h))
    assert status == -1                                            # neither W nor coefficients


@pytest.mark.parametrize("r_i", [0, 4])
def test_kv_append_scores_and_attention(env, r_i):
    """H = 16 heads of E = 16 dims on the 2048-slot ring (t = 8): the cache is built by appends,
    then q K^T and s V run against it."""
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    H, E, L = 16, 16, octx.prm.L
    lay = packing.KvLayout(octx.S, H, E, r_i)
    ntok = 13
    q, K, V, s = inputs.attention_inputs(7, H, 4, E, ntok)
    lv = L - 1                                   # cache level; appended vectors arrive at L
    kv = gctx.kv_create(H, E, lv, r_i=r_i)
    steps = lay.qk_steps() + lay.sv_steps() + lay.append_steps()
    assert sorted(set(kv.steps())) == sorted(set(steps))
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    ops = vmm.CkksOps(octx, okeys)

    # base masks: encoded once by the oracle; both sides derive every mask from them by the
    # exact Galois map on the integer coefficients
    def base(kind, level):
        m = np.zeros(octx.S)
        if kind == 0:
            m[:H * lay.t] = 1
        elif kind == 1:
            m[::lay.t] = 1
        else:
            m[[h * lay.t for h in range(H)]] = 1
        return octx.encode_coeffs(m, float(octx.mod[level]))

    bases = {0: base(0, lv - 1), 1: base(1, lv + 1), 2: base(2, lv + 1)}
    for kind, c in bases.items():
        kv.set_mask(kind, c)

    def omask(kind, shift_right, level):
        g = octx.galois(-shift_right)
        idx = octx.q_idx(level)
        coeff = octx.automorphism_coeff(octx.from_i64(bases[kind], idx), idx, g)
        from oracle.ckks import Pt
        return Pt(octx.ntt(coeff, idx), level, float(octx.mod[level]))

    # the rotated base masks are the layout's masks (checked on decoded slots)
    m = omask(2, lay.slot(3, 0, 5), lv + 1)
    dec = octx.decode_coeffs(np.array(octx.centred_coeffs(octx.intt(m.m, octx.q_idx(lv + 1)), 1), dtype=float) / m.scale)
    want = np.zeros(octx.S)
    want[[lay.slot(3, h, 5) for h in range(H)]] = 1
    assert np.abs(dec - want).max() < 1e-6

    okc, ovc = [], [None] * E
    for n in range(ntok):
        c, tau = n // lay.t, n % lay.t
        ok_new, gk_new = _enc_both(e, lay.pack_vec(K[n], tau), L, 100 + n)
        ov_new, gv_new = _enc_both(e, lay.pack_vec(V[n], tau), L, 500 + n)
        vmasks = [omask(2, lay.slot((c - k) % E, 0, tau) + lay.v_shift(k), lv + 1) for k in range(E)]
        vmm.kv_append(ops, lay, okc, ovc, n, ok_new, ov_new, omask(1, tau, lv + 1), vmasks)
        kv.append(gkeys, gk_new, gv_new)
    assert kv.tokens() == ntok
    for c in range(len(okc)):
        assert np.array_equal(kv.export(B.CM_QK, c), octx.canonical(okc[c]))
    for k in (0, 1, E - 1):
        assert np.array_equal(kv.export(B.CM_SV, k), octx.canonical(ovc[k]))

    oq, gq = _enc_both(e, lay.pack_vec(q), lv, 10)
    om = vmm.qk_scores(ops, lay, oq, okc, [omask(0, (c % E) * H * lay.t, lv - 1) for c in range(len(okc))])
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
    _same(e, om, gm)
    got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL

    os_, gs = _enc_both(e, lay.pack_scores(s), lv, 50)
    oa = vmm.score_times_v(ops, lay, os_, ovc)
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
    _same(e, oa, ga)
    assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


def test_kv_with_library_masks_decrypts_correctly(env):
    """The library's own mask encoder (no coefficients handed in)."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    H, E, L = 8, 32, octx.prm.L
    lay = packing.KvLayout(octx.S, H, E, 8)
    ntok = 11
    q, K, V, s = inputs.attention_inputs(9, H, 2, E, ntok)
    kv = gctx.kv_create(H, E, L - 1, r_i=8)
    gkeys = gctx.keygen_rotations(e["gsk"], kv.steps(), 2, with_relin=True)
    for n in range(ntok):
        tau = n % lay.t
        _, gk_new = _enc_both(e, lay.pack_vec(K[n], tau), L, 100 + n)
        _, gv_new = _enc_both(e, lay.pack_vec(V[n], tau), L, 500 + n)
        kv.append(gkeys, gk_new, gv_new)
    _, gq = _enc_both(e, lay.pack_vec(q), L - 1, 10)
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
    got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    _, gs = _enc_both(e, lay.pack_scores(s), L - 1, 50)
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
    assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL


@pytest.mark.parametrize("H,E,nk", [(16, 16, 3), (4, 64, 10), (2, 128, 2)])
def test_kv_qk_with_unrolled_ladders_matches_oracle_and_float64(env, H, E, nk):
    """q K^T with the sum over the head dims in the extended basis (CM_KV_UNROLLED_LADDERS): E = 16 is two
    runs of two ladder steps, 64 two runs of three, 128 runs of three, two and two; ten key ciphertexts
    make two batches (8 + 2).  Limbs against the oracle's form of it, scores against float64."""
    from oracle import packing, vmm
    from oracle.ckks import Pt
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    L = octx.prm.L
    lay = packing.KvLayout(octx.S, H, E)
    ntok = nk * lay.t - 2
    q, K, V, s = inputs.attention_inputs(17, H, max(1, H // 4), E, ntok)
    q = q * 0.3
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, unrolled_ladders=True)
    steps = vmm.qk_unrolled_steps(lay)
    assert set(steps) <= set(kv.steps())
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    m0 = np.zeros(octx.S)
    m0[:H * lay.t] = 1
    base = octx.encode_coeffs(m0, float(octx.mod[lv - 1]))
    kv.set_mask(0, base)

    def omask(c):
        idx = octx.q_idx(lv - 1)
        coeff = octx.automorphism_coeff(octx.from_i64(base, idx), idx, octx.galois(-(c % E) * H * lay.t))
        return Pt(octx.ntt(coeff, idx), lv - 1, float(octx.mod[lv - 1]))

    okc = []
    for c in range(nk):
        ok, gk = _enc_both(e, lay.pack_k(K, c), lv, 100 + c)
        okc.append(ok)
        kv.load(B.CM_QK, c, gk)
    kv.set_tokens(ntok)
    oq, gq = _enc_both(e, lay.pack_vec(q), lv, 10)
    om = vmm.qk_scores_unrolled(octx, okeys, lay, oq, okc, [omask(c) for c in range(nk)])
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
    _same(e, om, gm)
    got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    # twice in a row on the same buffers
    assert np.array_equal(gctx.ct_export(gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)), gctx.ct_export(gm))


@pytest.mark.parametrize("H,E,r_i", [(16, 16, 4), (16, 16, 0), (2, 128, 8)])
def test_kv_sv_with_unrolled_giant_steps_and_ladder_matches_oracle_and_float64(env, H, E, r_i):
    """scores V with CM_KV_UNROLLED_LADDERS: giant steps unrolled and the residue ladder in the extended
    basis; (2, 128, 8) has 16 giant-step groups, i.e. 15 rotations raised in two batches."""
    from oracle import packing, vmm
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    L = octx.prm.L
    lay = packing.KvLayout(octx.S, H, E, r_i)
    ntok = 3 * lay.t - 2
    q, K, V, s = inputs.attention_inputs(23, H, max(1, H // 4), E, ntok)
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, r_i=r_i, unrolled_ladders=True)
    steps = vmm.sv_unrolled_steps(lay)
    assert set(steps) <= set(kv.steps())
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    ovc = []
    for k in range(E):
        ov, gv = _enc_both(e, lay.pack_v(V, k), lv, 300 + k)
        ovc.append(ov)
        kv.load(B.CM_SV, k, gv)
    kv.set_tokens(ntok)
    os_, gs = _enc_both(e, lay.pack_scores(s), lv, 50)
    oa = vmm.score_times_v_unrolled(octx, okeys, lay, os_, ovc)
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
    _same(e, oa, ga)
    assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL
    assert np.array_equal(gctx.ct_export(gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)), gctx.ct_export(ga))


@pytest.mark.parametrize("ring,H,E,nk,shared", [
    ("config1", 16, 16, 3, 16),      # every rotation shared: no per-ciphertext ladder
    ("config1", 16, 16, 3, 4),       # two ladder steps per key ciphertext, three shared rotations
    ("config1", 4, 64, 10, 64),      # 63 shared rotations raised in eight batches; two batches of key ciphertexts
    ("config1", 4, 64, 10, 2),
    ("config1", 2, 128, 40, 128),    # enough products for the transform along the copy index (nk * shared >= 16 E)
    ("config1", 2, 128, 40, 64),     # ... with one ladder step left per key ciphertext
    ("config1", 4, 64, 20, 64),
    ("config1", 16, 16, 16, 16),     # the shortest transform that can pay (64 coefficients per workgroup)
    ("config1", 2, 256, 32, 128),    # 256 copies: 16 coefficients per workgroup, half of the rows written
    ("config1", 2, 128, 40, 16),     # more key ciphertexts than one LDS stage of the direct sums (32 + 8)
    ("wide", 4, 16, 5, 16),          # 54-bit primes: the integer form of the direct sums
    ("wide", 4, 16, 5, 2),
    ("wide", 2, 32, 20, 32),         # 54-bit primes through the transform
])
def test_kv_qk_with_shared_dim_rotations_matches_oracle_and_float64(env, ring, H, E, nk, shared):
    """q K^T with the copy mask applied before the last `shared` terms of the sum over the dims
    (cm_kv_set_shared_dims): limbs against the oracle's form of it, scores against float64, and the same
    message as the printed order."""
    from oracle import ckks, packing, params, vmm
    from oracle.ckks import Pt
    from paper_2602_11470_amd import inputs
    if ring == "wide":
        prm = params.toy(n=4096, q0_bits=58, qi_bits=54, scale_bits=54, name="wide")
        B = env["B"]
        gctx = B.Context(4096, 5, 1, 1, 58, 54, 60, 2.0 ** 54)
        octx = ckks.Context(prm)
        e = dict(B=B, octx=octx, gctx=gctx, osk=octx.keygen_secret(1), gsk=gctx.keygen_secret(1), prm=prm)
        assert [int(x) for x in gctx.moduli()] == [int(x) for x in octx.mod]
    else:
        e = env
    try:
        B, octx, gctx = e["B"], e["octx"], e["gctx"]
        L = octx.prm.L
        lay = packing.KvLayout(octx.S, H, E)
        ntok = nk * lay.t - 2
        q, K, V, s = inputs.attention_inputs(19, H, max(1, H // 4), E, ntok)
        q = q * 0.3
        lv = L - 1
        kv = gctx.kv_create(H, E, lv, unrolled_ladders=True, shared_dims=shared)
        steps = vmm.qk_shared_steps(lay, shared)
        assert set(steps) <= set(kv.steps())
        okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
        gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
        m0 = np.zeros(octx.S)
        m0[:H * lay.t] = 1
        base = octx.encode_coeffs(m0, float(octx.mod[lv - 1]))
        kv.set_mask(0, base)

        def omask(c):
            idx = octx.q_idx(lv - 1)
            coeff = octx.automorphism_coeff(octx.from_i64(base, idx), idx, octx.galois(-(c % E) * H * lay.t))
            return Pt(octx.ntt(coeff, idx), lv - 1, float(octx.mod[lv - 1]))

        okc = []
        for c in range(nk):
            ok, gk = _enc_both(e, lay.pack_k(K, c), lv, 100 + c)
            okc.append(ok)
            kv.load(B.CM_QK, c, gk)
        kv.set_tokens(ntok)
        oq, gq = _enc_both(e, lay.pack_vec(q), lv, 10)
        masks = [omask(b) for b in range(E)]
        om = vmm.qk_scores_shared(octx, okeys, lay, oq, okc, masks, shared)
        gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
        _same(e, om, gm)
        got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
        assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
        # twice in a row on the same buffers
        assert np.array_equal(gctx.ct_export(gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)), gctx.ct_export(gm))
        # back to the printed order on the same cache: the same scores
        kv.set_shared_dims(1)
        k1 = gctx.keygen_rotations(e["gsk"], kv.steps(), 2, with_relin=True)
        ref = gctx.decrypt(e["gsk"], gctx.vmm_kv(k1, kv, B.CM_QK, gq)).real
        assert np.abs(gctx.decrypt(e["gsk"], gm).real - ref).max() < 1e-6
    finally:
        if ring == "wide":
            e["gctx"].close()


def test_kv_shared_dims_rejects_other_caches_and_sizes(env):
    B, gctx = env["B"], env["gctx"]
    L = env["octx"].prm.L
    plain = gctx.kv_create(16, 16, L - 1)
    with pytest.raises(B.CachemirError) as ei:
        plain.set_shared_dims(4)
    assert ei.value.status == -1          # CM_E_INVAL: not an unrolled cache
    kv = gctx.kv_create(16, 16, L - 1, unrolled_ladders=True)
    for bad in (3, 32, 0):
        with pytest.raises(B.CachemirError) as ei:
            kv.set_shared_dims(bad)
        assert ei.value.status == -5      # CM_E_LAYOUT
    n0 = len(kv.steps())
    kv.set_shared_dims(16)
    assert {k * 16 * 8 for k in range(1, 16)} <= set(kv.steps())
    kv.set_shared_dims(1)
    assert len(kv.steps()) == n0


@pytest.mark.parametrize("r_i,unrolled", [(4, False), (0, False), (4, True), (8, True)])
def test_kv_key_index_appends_and_scores_match_oracle_and_float64(env, r_i, unrolled):
    """CM_KV_KEY_INDEX: one token group and five single tokens are appended; the K cache, the V cache and the
    key index limb for limb against the oracle; q K^T from the index (one level, no mask) limb for limb and
    against float64, for one query and for a query group; scores V unchanged."""
    from oracle import packing, vmm
    from oracle.ckks import Pt
    from paper_2602_11470_amd import inputs
    e = env
    B, octx, gctx = e["B"], e["octx"], e["gctx"]
    H, E, L = 16, 16, octx.prm.L
    lay = packing.KvLayout(octx.S, H, E, r_i)            # t = 8
    ntok = lay.t + 5
    q, K, V, s = inputs.attention_inputs(27, H, 4, E, ntok)
    q = q * 0.3
    lv = L - 1
    kv = gctx.kv_create(H, E, lv, r_i=r_i, unrolled_ladders=unrolled, key_index=True)
    sv_steps = vmm.sv_unrolled_steps(lay) if unrolled else lay.sv_steps()
    steps = sorted(set(lay.qk_steps()[:3]) | set(sv_steps) | set(lay.append_steps()) | set(lay.k_index_steps()))
    assert sorted(set(kv.steps())) == steps              # no rotation for the sum over the dims
    okeys = octx.keygen_rotations(e["osk"], steps, 2, with_relin=True)
    gkeys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
    ops = vmm.CkksOps(octx, okeys)
    ql = float(octx.mod[lv + 1])

    def base(kind):
        m = np.zeros(octx.S)
        if kind == 1:
            m[::lay.t] = 1
        elif kind == 2:
            m[[h * lay.t for h in range(H)]] = 1
        elif kind == 3:
            m[:] = 1
        else:
            m[:H * lay.t] = 1
        return octx.encode_coeffs(m, ql)

    bases = {k: base(k) for k in (1, 2, 3, 4)}
    for kind, c in bases.items():
        kv.set_mask(kind, c)

    def omask(kind, shift_right):
        idx = octx.q_idx(lv + 1)
        coeff = octx.automorphism_coeff(octx.from_i64(bases[kind], idx), idx, octx.galois(-shift_right))
        return Pt(octx.ntt(coeff, idx), lv + 1, ql)

    okc, ovc, oxc = [], [None] * E, [None] * E
    # group 0 at once
    kg = sum(lay.pack_vec(K[tau], tau) for tau in range(lay.t))
    vg = sum(lay.pack_vec(V[tau], tau) for tau in range(lay.t))
    ok_g, gk_g = _enc_both(e, kg, L, 90)
    ov_g, gv_g = _enc_both(e, vg, L, 91)
    vmm.kv_append_group(ops, lay, okc, ovc, 0, ok_g, ov_g, omask(3, 0),
                        [omask(4, lay.slot((0 - k) % E, 0, 0) + lay.v_shift(k)) for k in range(E)],
                        oxc, [omask(4, lay.slot((0 + (k // lay.r_i) * lay.r_i) % E, 0, 0)) for k in range(E)])
    kv.append_group(gkeys, gk_g, gv_g)
    for n in range(lay.t, ntok):
        c, tau = n // lay.t, n % lay.t
        ok_new, gk_new = _enc_both(e, lay.pack_vec(K[n], tau), L, 100 + n)
        ov_new, gv_new = _enc_both(e, lay.pack_vec(V[n], tau), L, 500 + n)
        vmasks = [omask(2, lay.slot((c - k) % E, 0, tau) + lay.v_shift(k)) for k in range(E)]
        xmasks = [omask(2, lay.slot((c + (k // lay.r_i) * lay.r_i) % E, 0, tau)) for k in range(E)]
        vmm.kv_append(ops, lay, okc, ovc, n, ok_new, ov_new, omask(1, tau), vmasks, oxc, xmasks)
        kv.append(gkeys, gk_new, gv_new)
    assert kv.tokens() == ntok
    for c in range(len(okc)):
        assert np.array_equal(kv.export(B.CM_QK, c), octx.canonical(okc[c]))
    for k in range(E):
        assert np.array_equal(kv.export(B.CM_KV_INDEX, k), octx.canonical(oxc[k])), k
    assert np.array_equal(kv.export(B.CM_SV, 3), octx.canonical(ovc[3]))
    # the index decrypts to the layout
    for k in (0, 5, E - 1):
        assert np.abs(octx.decrypt(e["osk"], oxc[k]).real - lay.pack_k_index(K, k)).max() < TOL

    sv = (lambda c, x: vmm.score_times_v_unrolled(octx, okeys, lay, c, x, reduce=False)) if unrolled else None
    oq, gq = _enc_both(e, lay.pack_vec(q), lv, 10)
    om = vmm.qk_scores_indexed(ops, lay, oq, oxc, sv=sv)
    gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gq)
    assert gm.level == lv - 1
    _same(e, om, gm)
    got = lay.unpack_scores(gctx.decrypt(e["gsk"], gm).real, ntok)
    assert np.abs(got - np.einsum("he,nhe->hn", q, K)).max() < TOL
    # a query group: query tau against the keys of residue tau
    Q = np.random.default_rng(5).normal(size=(lay.t, H, E)) * 0.3
    oqg, gqg = _enc_both(e, sum(lay.pack_vec(Q[tau], tau) for tau in range(lay.t)), lv, 11)
    og = vmm.qk_scores_indexed(ops, lay, oqg, oxc, replicate=False, sv=sv)
    gg = gctx.vmm_kv(gkeys, kv, B.CM_QK_GROUP, gqg)
    _same(e, og, gg)
    gotg = lay.unpack_scores(gctx.decrypt(e["gsk"], gg).real, ntok)
    for n in range(ntok):
        assert np.abs(gotg[:, n] - np.einsum("he,he->h", Q[n % lay.t], K[n])).max() < TOL
    # scores V as before
    os_, gs = _enc_both(e, lay.pack_scores(s), lv, 50)
    oa = vmm.score_times_v_unrolled(octx, okeys, lay, os_, ovc) if unrolled else vmm.score_times_v(ops, lay, os_, ovc)
    ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
    _same(e, oa, ga)
    # load / export of an index ciphertext; not available without the index
    kv.load(B.CM_KV_INDEX, 2, gctx.level_drop(gk_g, lv))
    assert np.array_equal(kv.export(B.CM_KV_INDEX, 2), gctx.ct_export(gctx.level_drop(gk_g, lv)))
    plain = gctx.kv_create(H, E, lv, r_i=r_i)
    with pytest.raises(B.CachemirError) as ei:
        plain.export(B.CM_KV_INDEX, 0)
    assert ei.value.status == -1


@pytest.mark.parametrize("r_i", [4, 0])
def test_kv_sv_on_54_bit_primes_matches_oracle(env, r_i):
    """scores V on a ring whose primes are too long for the FP64 forms: the integer form of the summed tensor products."""
    from oracle import ckks, packing, params, vmm
    from paper_2602_11470_amd import inputs
    B = env["B"]
    prm = params.toy(n=4096, q0_bits=58, qi_bits=54, scale_bits=54, name="wide")
    gctx = B.Context(4096, 5, 1, 1, 58, 54, 60, 2.0 ** 54)
    try:
        octx = ckks.Context(prm)
        e = dict(B=B, octx=octx, gctx=gctx, osk=octx.keygen_secret(1), gsk=gctx.keygen_secret(1), prm=prm)
        H, E, L = 4, 16, prm.L
        lay = packing.KvLayout(octx.S, H, E, r_i)        # t = 32
        ntok = 2 * lay.t + 3
        q, K, V, s = inputs.attention_inputs(33, H, 1, E, ntok)
        lv = L - 1
        kv = gctx.kv_create(H, E, lv, r_i=r_i)
        okeys = octx.keygen_rotations(e["osk"], lay.sv_steps(), 2, with_relin=True)
        gkeys = gctx.keygen_rotations(e["gsk"], lay.sv_steps(), 2, with_relin=True)
        ovc = []
        for k in range(E):
            ov, gv = _enc_both(e, lay.pack_v(V, k), lv, 300 + k)
            ovc.append(ov)
            kv.load(B.CM_SV, k, gv)
        kv.set_tokens(ntok)
        os_, gs = _enc_both(e, lay.pack_scores(s), lv, 50)
        oa = vmm.score_times_v(vmm.CkksOps(octx, okeys), lay, os_, ovc)
        ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, gs)
        _same(e, oa, ga)
        assert np.abs(lay.unpack_vec(gctx.decrypt(e["gsk"], ga).real) - np.einsum("hn,nhe->he", s, V)).max() < TOL
    finally:
        gctx.close()


def test_keys_with_stored_uniform_halves_give_the_same_ciphertexts(env):
    """CM_OPT_EVK_STORED_A keeps a_j in device memory instead of regenerating it in the kernels: the same
    residues, so every kernel of the inner-product family gives bit for bit what it gives with the default keys
    -- the single one (rotate), the source-stationary one (hoisted baby steps), the batched one (unrolled giant
    steps and ladders of the packed product), the shared-key and multi-key ones (q K^T with unrolled ladders)."""
    from paper_2602_11470_amd import inputs
    e = env
    B, gctx = e["B"], e["gctx"]
    L = gctx.L
    x, W = inputs.vmm_inputs(31, 256, 256, "uniform", 0.05)
    gplan = gctx.vmm_plan(256, 256, W=W, level=L, unrolled_ladders=True)
    H, E = 4, 64
    kv_flags = dict(unrolled_ladders=True)
    rng = np.random.default_rng(5)
    slots = [rng.uniform(-1, 1, gctx.S) for _ in range(12)]

    def run(stored):
        gctx.set_option(B.CM_OPT_EVK_STORED_A, stored)
        try:
            kv = gctx.kv_create(H, E, L - 1, **kv_flags)
            steps = sorted(set(gplan.steps()) | set(kv.steps()) | {7})
            keys = gctx.keygen_rotations(e["gsk"], steps, 2, with_relin=True)
            enc = lambda i, lv: gctx.level_drop(gctx.encrypt(e["gsk"], gctx.encode(slots[i], L), 40 + i), lv)
            out = [gctx.ct_export(gctx.rotate(keys, enc(0, L), 7))]
            out += [gctx.ct_export(c) for c in gctx.rotate_hoisted(keys, enc(1, L - 2), gplan.steps()[:5])]
            out.append(gctx.ct_export(gctx.vmm_pt(keys, gplan, enc(2, L))))
            for c in range(10):
                kv.load(B.CM_QK, c, enc(c % 6 + 3, L - 1))
            kv.set_tokens(10 * (gctx.S // (H * E)))
            out.append(gctx.ct_export(gctx.vmm_kv(keys, kv, B.CM_QK, enc(9, L - 1))))
            out.append(keys.export(7, False, 2, 1))
            return out
        finally:
            gctx.set_option(B.CM_OPT_EVK_STORED_A, 0)

    ref, got = run(0), run(1)
    assert len(ref) == len(got)
    for a, b in zip(ref, got):
        assert np.array_equal(a, b)
