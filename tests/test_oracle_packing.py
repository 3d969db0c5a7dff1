"""Pins for the packing layer: the paper's printed toy layouts and operation counts, and the
plain float64 products, all on slot vectors without cryptography."""
import numpy as np
import pytest

from oracle import packing, vmm


def _tokens(line):
    return line.split()


def _sym(vals, names):
    """Map numeric slot vector back to the symbols of the fixture (0 stays '0')."""
    inv = {v: k for k, v in names.items()}
    return [inv.get(float(v), "0" if v == 0 else "?") for v in vals]


def test_toy_vmm_layouts_of_section_4_1(golden):
    g = golden("paper_toy_layouts.txt")
    names = {f"a{i}": float(i + 1) for i in range(4)}
    plan = packing.make_plan(8, 4, 4)
    c = plan.pack_input([names[f"a{i}"] for i in range(4)])
    assert _sym(c, names) == _tokens(g["vmm_input"])
    ops = vmm.SlotOps()
    for r in plan.pre_steps:
        c = ops.add(c, ops.rotate(c, r))
    assert _sym(c, names) == _tokens(g["vmm_preprocessed"])
    ops = vmm.SlotOps()
    rng = np.random.default_rng(0)
    x, W = rng.normal(size=4), rng.normal(size=(4, 4))
    y = vmm.vmm_pt(ops, plan, plan.pack_input(x), plan.diagonals(W))
    assert ops.rotations == int(g["vmm_rotations"]) == plan.n_rotations
    assert np.allclose(plan.unpack_output(y), x @ W, atol=1e-12)


def test_rotation_and_multiplication_counts_of_tables_2_and_4(golden):
    g = golden("paper_op_counts.txt")
    for d, key in ((4096, "rotations_d4096"), (2048, "rotations_d2048"), (1024, "rotations_d768")):
        plan = packing.make_plan(32768, d, d)
        assert plan.n_rotations == int(g[key])
        assert len(plan.all_steps()) - (plan.r_o > 1) + max(plan.r_o - 1, 0) == plan.n_rotations
    plan = packing.make_plan(32768, 4096, 4096)
    assert plan.M == plan.r_i * plan.r_o == int(g["ptct_mults_d4096"])
    lay = packing.KvLayout(32768, 32, 128)
    assert lay.capacity == int(g["score_capacity_llama3_8b"])
    assert lay.E == int(g["v_cts_llama3_8b"])


def test_counts_by_running_the_algorithm_at_table_2_shape():
    """Instrumented run on plain slot vectors at (S, d) = (32768, 4096): 52 rotations and 512
    plaintext products, and the result is x W."""
    plan = packing.make_plan(32768, 4096, 4096)
    rng = np.random.default_rng(1)
    x, W = rng.normal(size=4096), rng.normal(0, 0.02, (4096, 4096))
    ops = vmm.SlotOps()
    y = vmm.vmm_pt(ops, plan, plan.pack_input(x), plan.diagonals(W))
    assert (ops.rotations, ops.pt_mults) == (52, 512)
    assert np.abs(plan.unpack_output(y) - x @ W).max() < 1e-11


@pytest.mark.parametrize("S,d_in,d_out,r_i", [
    (8, 4, 4, None), (64, 8, 8, 1), (64, 8, 8, None), (2048, 64, 64, None), (256, 32, 32, 4),
    (64, 8, 32, None), (64, 32, 8, None), (2048, 64, 256, None), (2048, 256, 64, 2),
    (1024, 128, 32, None), (1024, 32, 128, 2), (512, 16, 32, None)])
def test_packed_product_equals_float64_product(S, d_in, d_out, r_i):
    plan = packing.make_plan(S, d_in, d_out, r_i)
    rng = np.random.default_rng(S + d_in)
    x, W = rng.normal(size=d_in), rng.normal(size=(d_in, d_out))
    ops = vmm.SlotOps()
    y = vmm.vmm_pt(ops, plan, plan.pack_input(x), plan.diagonals(W))
    assert np.abs(plan.unpack_output(y) - x @ W).max() < 1e-12
    assert ops.rotations == plan.n_rotations and ops.pt_mults == plan.M
    # the printed count: log t + log t' + (r_i - 1) + (r_o - 1)
    lg = lambda v: v.bit_length() - 1
    assert plan.n_rotations == lg(plan.t) + lg(plan.tp) + plan.r_i + plan.r_o - 2
    assert plan.r_i * plan.r_o * plan.tp == plan.d


@pytest.mark.parametrize("tau", [1, 2, 5, 7])
def test_customised_residue_output(tau):
    plan = packing.make_plan(64, 8, 8, tau=tau)
    rng = np.random.default_rng(tau)
    x, W = rng.normal(size=8), rng.normal(size=(8, 8))
    y = vmm.vmm_pt(vmm.SlotOps(), plan, plan.pack_input(x), plan.diagonals(W))
    assert np.allclose(y[tau::8], x @ W, atol=1e-12)
    assert all(s == plan.out_slot(c) for c, s in enumerate(range(tau, 64, 8)))


def test_k_cache_toy_layouts_of_section_5_1(golden):
    g = golden("paper_toy_layouts.txt")
    lay = packing.KvLayout(8, 1, 4)
    assert lay.t == 2
    K = np.array([[[10 * i + j + 100 for j in range(4)]] for i in range(6)], dtype=float)
    names = {f"k{i}{j}": K[i, 0, j] for i in range(6) for j in range(4)}
    assert _sym(lay.pack_k(K[:5], 0), names) == _tokens(g["k_cache_ct0"])
    q = np.array([[1., 2., 3., 4.]])
    qn = {f"q{j}": q[0, j] for j in range(4)}
    ops = vmm.SlotOps()
    cq = lay.pack_vec(q)
    for i in range(1):
        cq = ops.add(cq, ops.rotate(cq, -(1 << i)))
    assert _sym(cq, qn) == _tokens(g["q_replicated"])
    # replicated map of ciphertext 0
    p = cq * lay.pack_k(K[:5], 0)
    for i in range(2):
        p = p + np.roll(p, -(1 << i) * lay.t)
    m = K[:5, 0, :] @ q[0]
    mn = {f"m{i}": m[i] for i in range(5)}
    assert _sym(p, mn) == _tokens(g["map_replicated"])
    assert [str(int(v)) for v in lay.qk_mask(0)] == _tokens(g["qk_mask_ct0"])
    packed = vmm.qk_scores(vmm.SlotOps(), lay, lay.pack_vec(q),
                           [lay.pack_k(K[:5], c) for c in range(3)],
                           [lay.qk_mask(c) for c in range(3)])
    assert _sym(packed, mn) == _tokens(g["map_packed_5_tokens"])
    # appended token 5 sits on residue 1
    assert _sym(lay.pack_vec(K[5], tau=5 % lay.t), names) == _tokens(g["k_append_tok5"])


def test_multi_head_toy_layouts_of_section_5_3(golden):
    g = golden("paper_toy_layouts.txt")
    lay = packing.KvLayout(8, 2, 2)           # d = 4, H = 2, t = 2
    # the paper's k_ij = dimension j of token i; head h owns dims {2h, 2h+1}
    Kflat = np.array([[10 * i + j + 100 for j in range(4)] for i in range(2)], dtype=float)
    K = Kflat.reshape(2, 2, 2)                # [token, h, e]
    names = {f"k{i}{j}": Kflat[i, j] for i in range(2) for j in range(4)}
    assert _sym(lay.pack_k(K, 0), names) == _tokens(g["mh_k_cache_ct0"])
    q = np.array([[1., 2.], [3., 5.]])
    m = np.einsum("he,nhe->hn", q, K)
    mn = {f"m{n}h{h}": m[h, n] for h in range(2) for n in range(2)}
    packed = vmm.qk_scores(vmm.SlotOps(), lay, lay.pack_vec(q), [lay.pack_k(K, 0)],
                           [lay.qk_mask(0)])
    assert _sym(packed, mn) == _tokens(g["mh_map"])
    att = np.array([[7., 8.], [9., 11.]])     # a_e^h
    an = {f"a{e}h{h}": att[h, e] for h in range(2) for e in range(2)}
    assert _sym(lay.pack_vec(att), an) == _tokens(g["mh_att"])


@pytest.mark.parametrize("S,H,E,r_i,ntok", [(8, 1, 4, 0, 5), (256, 4, 8, 0, 61), (256, 4, 8, 4, 64),
                                            (512, 2, 16, 4, 100), (64, 4, 16, 2, 9)])
def test_attention_products_equal_float64_einsum(S, H, E, r_i, ntok):
    lay = packing.KvLayout(S, H, E, r_i)
    assert ntok <= lay.capacity
    rng = np.random.default_rng(S + ntok)
    q, K, V = rng.normal(size=(H, E)), rng.normal(size=(ntok, H, E)), rng.normal(size=(ntok, H, E))
    nk = -(-ntok // lay.t)
    ops = vmm.SlotOps()
    m = vmm.qk_scores(ops, lay, lay.pack_vec(q), [lay.pack_k(K, c) for c in range(nk)],
                      [lay.qk_mask(c) for c in range(nk)])
    assert np.abs(lay.unpack_scores(m, ntok) - np.einsum("he,nhe->hn", q, K)).max() < 1e-12
    lg = lambda v: v.bit_length() - 1
    assert ops.ct_mults == nk and ops.rotations == lg(lay.t) + nk * lg(E)
    # unused score slots are zero, so the score ciphertext feeds the next product directly
    assert np.count_nonzero(m) <= H * ntok
    s = rng.uniform(size=(H, ntok))
    s /= s.sum(axis=1, keepdims=True)
    ops = vmm.SlotOps()
    a = vmm.score_times_v(ops, lay, lay.pack_scores(s), [lay.pack_v(V, k) for k in range(E)])
    assert np.abs(lay.unpack_vec(a) - np.einsum("hn,nhe->he", s, V)).max() < 1e-12
    assert ops.ct_mults == E
    assert ops.rotations == (lay.r_i - 1) + (lay.r_o - 1) + lg(lay.t)
    assert sorted(set(lay.sv_steps())) == sorted(set(
        [j * H * lay.t for j in range(1, lay.r_i)] + [1 << l for l in range(lg(lay.t))] +
        ([lay.r_i * H * lay.t] if lay.r_o > 1 else [])))


@pytest.mark.parametrize("r_i", [0, 2])
def test_cache_append_builds_the_same_cache_as_packing_all_tokens(r_i):
    lay = packing.KvLayout(128, 2, 8, r_i)
    rng = np.random.default_rng(3)
    ntok = 21
    K, V = rng.normal(size=(ntok, 2, 8)), rng.normal(size=(ntok, 2, 8))
    kc, vc = [], [None] * lay.E
    for n in range(ntok):
        tau = n % lay.t
        junk = 0.5 * lay.residue_mask((tau + 1) % lay.t)       # partial sums on other residues
        vmm.kv_append(vmm.SlotOps(), lay, kc, vc, n, lay.pack_vec(K[n], tau) + junk,
                      lay.pack_vec(V[n], tau) + junk, lay.residue_mask(tau),
                      [lay.v_append_mask(k, n) for k in range(lay.E)])
    assert len(kc) == -(-ntok // lay.t)
    for c in range(len(kc)):
        assert np.array_equal(kc[c], lay.pack_k(K, c))
    for k in range(lay.E):
        assert np.array_equal(vc[k], lay.pack_v(V, k))
