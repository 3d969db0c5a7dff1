"""Benchmark configuration 5 on the GPU: the linear path of one Llama-3-8B-shaped decoder layer per token on
the ring of 36 ciphertext primes + 6 special primes (6 digits of 6), four decode steps, every stage
decrypted and compared with float64 within 1e-4."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def ring5():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from oracle import params
    from paper_2602_11470_amd import binding as B
    gctx = B.llama_ring(36, 6)
    yield B, gctx, params.llama_ring(36, 6)
    gctx.close()


def _rope_ref(v, n, E):
    out = np.empty_like(v)
    for m in range(E // 2):
        th = n * 10000.0 ** (-2.0 * m / E)
        out[:, 2 * m] = v[:, 2 * m] * np.cos(th) - v[:, 2 * m + 1] * np.sin(th)
        out[:, 2 * m + 1] = v[:, 2 * m + 1] * np.cos(th) + v[:, 2 * m] * np.sin(th)
    return out


def test_config5_four_decode_steps_of_a_layers_linear_path(ring5):
    """Four decode steps of one layer: q / k / v projections of the token (one call: the preprocess rotations
    and the hoisted baby steps are shared, cm_vmm_pt_multi; 8 KV heads replicated to 32 by repeating weight
    columns, columns ordered as the cache wants them), the rotary embedding of q and k with the extraction fused
    (Sec. 4.2), append of the encrypted k / v to a cache that already holds 16 tokens, q K^T against the cache,
    scores V, the output projection, and the MLP: gate and up (4096 -> 14336, padded to 16384, one shared-baby-
    step call) and down (14336 -> 4096).  The non-linear layers between these stages (softmax, normalisations,
    SiLU) are outside this path: where the model has one, the next stage starts from a fresh encryption of the
    float64 value, at the paper's operating level for that stage (Table 5)."""
    from oracle import packing
    from paper_2602_11470_amd import inputs
    B, gctx, prm = ring5
    H, E, d, L = 32, 128, 4096, gctx.L
    dm, real = 16384, 14336
    lay = packing.KvLayout(gctx.S, H, E, 16)
    t = lay.t
    rng = np.random.default_rng(5)
    Wq, Wo = rng.normal(0, 0.02, (d, d)), rng.normal(0, 0.02, (d, d))
    Wk8, Wv8 = rng.normal(0, 0.02, (d, 8 * E)), rng.normal(0, 0.02, (d, 8 * E))
    Wg, Wu, Wd = np.zeros((d, dm)), np.zeros((d, dm)), np.zeros((dm, d))
    Wg[:, :real], Wu[:, :real] = rng.normal(0, 0.02, (d, real)), rng.normal(0, 0.02, (d, real))
    Wd[:real, :] = rng.normal(0, 0.02, (real, d))
    # column a = e*H + h of the packed weights is column [h, e] of the model's (KV head h // 4)
    a = np.arange(d)
    e_of, h_of = a // H, a % H
    Wq_p = Wq[:, h_of * E + e_of]
    Wk_p, Wv_p = Wk8[:, (h_of // 4) * E + e_of], Wv8[:, (h_of // 4) * E + e_of]
    Wo_p = Wo[h_of * E + e_of, :]                      # rows follow the attention output layout
    gsk = gctx.keygen_secret(1)
    cache_lv = L - 3                     # projection, rotary embedding, append mask: one level each
    mlp_lv, down_lv = 4, 2               # the MLP at low levels (the paper runs up / gate at 3, down at 1)
    kv = gctx.kv_create(H, E, cache_lv, r_i=16)
    plan_q = gctx.vmm_plan(d, d, W=Wq_p, level=L, unrolled_ladders=True)
    plan_o = gctx.vmm_plan(d, d, W=Wo_p, level=cache_lv - 2, unrolled_ladders=True)
    plan_g = gctx.vmm_plan(d, dm, W=Wg, level=mlp_lv, unrolled_ladders=True)
    plan_u = gctx.vmm_plan(d, dm, W=Wu, level=mlp_lv, unrolled_ladders=True)
    plan_d = gctx.vmm_plan(dm, d, W=Wd, level=down_lv, unrolled_ladders=True)
    oplan_up, oplan_down = packing.make_plan(gctx.S, d, dm), packing.make_plan(gctx.S, dm, d)
    residue0 = np.zeros(gctx.S)
    residue0[::t] = 1.0

    def extract(ct):
        """Keep residue 0 of every block: mask encoded at the scale of the prime the rescale removes."""
        mask = gctx.encode(residue0, ct.level, float(prm.moduli[ct.level]), mont=True)
        return gctx.rescale(gctx.mul_pt(ct, mask))
    steps = set(kv.steps()) | set(plan_q.steps()) | set(plan_o.steps()) | {H * t, -H * t}
    for p in (plan_g, plan_u, plan_d):
        steps |= set(p.steps())
    # the k / v plans of a token differ from the q plan only in the residue their reduce ladder lands on
    from oracle import vmm as ovmm
    for tau in range(4):
        for grp in ovmm.ladder_groups(packing.make_plan(gctx.S, d, d, tau=tau).reduce_steps):
            steps |= set(grp)
    gkeys = gctx.keygen_rotations(gsk, sorted(steps), 2, with_relin=True)
    enc = lambda slots, level, seed, scale=0.0: gctx.level_drop(
        gctx.encrypt(gsk, gctx.encode(slots, L, scale), seed), level)
    n0 = 16
    _, K, V, _ = inputs.attention_inputs(4, H, 8, E, n0)
    # a cache holds one scale: the tokens already there carry the scale a projection leaves
    proj_scale = prm.scale * prm.scale / float(prm.moduli[L])
    for c in range(n0 // t):
        kv.load(B.CM_QK, c, enc(lay.pack_k(K, c), cache_lv, 100 + c, proj_scale))
    for k in range(E):
        kv.load(B.CM_SV, k, enc(lay.pack_v(V, k), cache_lv, 300 + k, proj_scale))
    kv.set_tokens(n0)
    K, V = list(K), list(V)
    worst = {}

    def close(name, got, want):
        err = float(np.abs(got - want).max())
        worst[name] = max(worst.get(name, 0.0), err)
        assert err < TOL, (name, err, worst)

    for step in range(4):
        n = n0 + step
        tau = n % t
        x = rng.normal(size=d)
        slots = np.zeros(gctx.S)
        slots[::t] = x
        gx = enc(slots, L, 500 + step)
        # q, k, v of the token in one call; k and v land on residue tau, ready for the append
        plan_k = gctx.vmm_plan(d, d, W=Wk_p, level=L, tau=tau, unrolled_ladders=True)
        plan_v = gctx.vmm_plan(d, d, W=Wv_p, level=L, tau=tau, unrolled_ladders=True)
        assert set(plan_k.steps()) <= steps
        gq, gk, gv = gctx.vmm_pt_multi(gkeys, [plan_q, plan_k, plan_v], gx)
        del plan_k, plan_v
        k_ref = _rope_ref((x @ Wk8).reshape(8, E).repeat(4, axis=0), n, E)          # [h, e]
        v_ref = (x @ Wv8).reshape(8, E).repeat(4, axis=0)
        gk = gctx.rope_apply(gkeys, gctx.rope(H, E, L - 1, n, tau), gk)             # level L-2, other slots clean
        close("k", lay.unpack_vec(gctx.decrypt(gsk, gk).real, tau), k_ref)
        kv.append(gkeys, gk, gctx.level_drop(gv, L - 2))
        K.append(k_ref), V.append(v_ref)
        assert kv.tokens() == n + 1
        gq = gctx.rope_apply(gkeys, gctx.rope(H, E, L - 1, n, 0), gq)
        q_ref = _rope_ref((x @ Wq).reshape(H, E), n, E)
        close("q", lay.unpack_vec(gctx.decrypt(gsk, gq).real), q_ref)
        gm = gctx.vmm_kv(gkeys, kv, B.CM_QK, gctx.level_drop(gq, cache_lv))
        Ka, Va = np.stack(K), np.stack(V)
        m_ref = np.einsum("he,nhe->hn", q_ref, Ka)
        close("qk", lay.unpack_scores(gctx.decrypt(gsk, gm).real, n + 1), m_ref)
        sc = np.abs(m_ref)
        sc /= sc.sum(axis=1, keepdims=True)
        ga = gctx.vmm_kv(gkeys, kv, B.CM_SV, enc(lay.pack_scores(sc), cache_lv, 700 + step))
        att_ref = np.einsum("hn,nhe->he", sc, Va)
        close("sv", lay.unpack_vec(gctx.decrypt(gsk, ga).real), att_ref)
        gy = gctx.vmm_pt(gkeys, plan_o, extract(ga))
        y_ref = att_ref.reshape(-1) @ Wo
        close("o", gctx.decrypt(gsk, gy).real[::t], y_ref)
        # MLP: gate and up share the input (one call), down takes the 16384-vector at interval 2
        hin = x + y_ref                                                           # stands for the normalised residual
        slots[::t] = hin
        gh = enc(slots, mlp_lv, 800 + step)
        gg, gu = gctx.vmm_pt_multi(gkeys, [plan_g, plan_u], gh)
        gate_ref, up_ref = hin @ Wg, hin @ Wu
        close("gate", oplan_up.unpack_output(gctx.decrypt(gsk, gg).real), gate_ref)
        close("up", oplan_up.unpack_output(gctx.decrypt(gsk, gu).real), up_ref)
        act = gate_ref / (1.0 + np.exp(-gate_ref)) * up_ref
        gd = gctx.vmm_pt(gkeys, plan_d, enc(oplan_down.pack_input(act), down_lv, 900 + step))
        close("down", gctx.decrypt(gsk, gd).real[::t], act @ Wd)
    print("config 5, worst max-abs errors over four steps:", {k: f"{v:.2e}" for k, v in worst.items()})
