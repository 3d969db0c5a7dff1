"""GPU parity of the encrypted-cache path at the benchmark's full size (ring n = 2^16, 24 + 4 primes,
Llama-3-8B attention shapes): cache appends (one token, a token group), q K^T (printed order and the form
the attention workload of bench.py times) and scores V (printed order and unrolled) against results the
ORACLE wrote (tests/golden/kv_full_size.txt, by tests/golden/make_kv_full_size_golden.py).  At this ring
size the library runs code the small-ring limb tests never reach: the masked products formed inside the
rescale's transform, the ModDown / rescale tails fused into the forward transform, the rescale that feeds the
last limb's residues to the other limbs' transforms without a reduction pass, and the masked sums through the
transform along the copy index."""
import hashlib
import importlib.util
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _mk():
    spec = importlib.util.spec_from_file_location(
        "mk_kv", os.path.join(os.path.dirname(__file__), "golden", "make_kv_full_size_golden.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    return mk


@pytest.fixture(scope="module")
def scene():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2602_11470_amd import binding as B
    mk = _mk()
    gctx = B.llama_ring(24, 4)
    gsk = gctx.keygen_secret(mk.SEED_SK)
    gkeys = gctx.keygen_rotations(gsk, mk.all_steps(gctx.S), mk.SEED_EVK, with_relin=True)
    yield dict(B=B, mk=mk, gctx=gctx, gsk=gsk, gkeys=gkeys)
    del gkeys
    gctx.close()


def _enc(s, seed, level):
    gctx, mk = s["gctx"], s["mk"]
    ct = gctx.encrypt(s["gsk"], gctx.pt_from_coeffs(mk.poly(gctx.n, seed), gctx.L, gctx.scale), 1000 + seed)
    return gctx.level_drop(ct, level)


def _cache(s, **flags):
    """A cache with the scenario's integer masks, after the group append and the two single appends."""
    gctx, mk = s["gctx"], s["mk"]
    L = gctx.L
    kv = gctx.kv_create(mk.H, mk.E, L - 1, r_i=mk.R_I, **flags)
    assert set(kv.steps()) <= set(mk.all_steps(gctx.S))
    for kind, seed in mk.MASK_SEEDS.items():
        kv.set_mask(kind, mk.poly(gctx.n, seed))
    kv.append_group(s["gkeys"], _enc(s, mk.GROUP_SEEDS[0], L), _enc(s, mk.GROUP_SEEDS[1], L))
    for tok in mk.TOKENS:
        kv.append(s["gkeys"], _enc(s, 100 + tok, L), _enc(s, 500 + tok, L))
    assert kv.tokens() == 10
    return kv


def _check(golden, name, can):
    g = golden("kv_full_size.txt")
    assert list(can.shape) == [int(v) for v in g[f"{name}_shape"].split()], name
    for c in range(can.shape[0]):
        for l in (0, can.shape[1] - 1):
            assert [int(v) for v in can[c, l, :4]] == [int(v) for v in g[f"{name}_head_{c}_{l}"].split()], (name, c, l)
    assert hashlib.sha256(np.ascontiguousarray(can).tobytes()).hexdigest() == g[f"{name}_sha256"], name


def test_appends_and_printed_order_products_equal_the_oracle(scene, golden):
    s = scene
    B, gctx, mk = s["B"], s["gctx"], s["mk"]
    kv = _cache(s)
    for c in range(2):
        _check(golden, f"K{c}", kv.export(B.CM_QK, c))
    hv = hashlib.sha256()
    for k in range(mk.E):
        can = kv.export(B.CM_SV, k)
        hv.update(can.tobytes())
        if k in (0, 17, mk.E - 1):
            _check(golden, f"V{k}", can)
    assert hv.hexdigest() == golden("kv_full_size.txt")["V_all_sha256"]
    lv = gctx.L - 1
    gm = gctx.vmm_kv(s["gkeys"], kv, B.CM_QK, _enc(s, mk.SEED_Q, lv))
    assert gm.level == lv - 2
    _check(golden, "qk_printed", gctx.ct_export(gm))
    ga = gctx.vmm_kv(s["gkeys"], kv, B.CM_SV, _enc(s, mk.SEED_S, lv))
    assert ga.level == lv - 1
    _check(golden, "sv_printed", gctx.ct_export(ga))


def test_the_attention_workloads_form_equals_the_oracle(scene, golden):
    """Unrolled ladders, copy mask in front of all 128 terms of the sum over the dims, 16 K ciphertexts (the
    masked sums go through the transform along the copy index, as with the workload's 128)."""
    s = scene
    B, gctx, mk = s["B"], s["gctx"], s["mk"]
    kv = _cache(s, unrolled_ladders=True, shared_dims=mk.SHARED)
    lv = gctx.L - 1
    ga = gctx.vmm_kv(s["gkeys"], kv, B.CM_SV, _enc(s, mk.SEED_S, lv))
    _check(golden, "sv_unrolled", gctx.ct_export(ga))
    for c in mk.LOADED_K:
        kv.load(B.CM_QK, c, _enc(s, 200 + c, lv))
    kv.set_tokens(16 * 8)
    gm = gctx.vmm_kv(s["gkeys"], kv, B.CM_QK, _enc(s, mk.SEED_Q, lv))
    _check(golden, "qk_shared", gctx.ct_export(gm))


def test_stored_uniform_halves_give_the_same_ciphertexts(scene):
    """CM_OPT_EVK_STORED_A: the kernels read a_j instead of regenerating it -- the same residues, so a rotation,
    hoisted rotations and a packed product are bit for bit what the default keys give."""
    s = scene
    B, gctx = s["B"], s["gctx"]
    steps = [7, 2048, 64, -4096]
    x = _enc(s, 77, gctx.L)
    ref_keys = gctx.keygen_rotations(s["gsk"], steps, 9, with_relin=True)
    ref_rot = gctx.ct_export(gctx.rotate(ref_keys, x, 7))
    ref_h = [gctx.ct_export(c) for c in gctx.rotate_hoisted(ref_keys, x, steps)]
    ref_b = ref_keys.export(64, False, 3, 0), ref_keys.export(64, False, 3, 1)
    gctx.set_option(B.CM_OPT_EVK_STORED_A, 1)
    try:
        with pytest.raises(B.CachemirError):                   # keys of the other kind are refused, not misread
            gctx.rotate(ref_keys, x, 7)
        keys = gctx.keygen_rotations(s["gsk"], steps, 9, with_relin=True)
        assert np.array_equal(keys.export(64, False, 3, 0), ref_b[0]) and np.array_equal(keys.export(64, False, 3, 1), ref_b[1])
        assert np.array_equal(gctx.ct_export(gctx.rotate(keys, x, 7)), ref_rot)
        for got, want in zip(gctx.rotate_hoisted(keys, x, steps), ref_h):
            assert np.array_equal(gctx.ct_export(got), want)
        sq = gctx.rescale(gctx.relinearize(keys, gctx.mul_ct(x, x)))
    finally:
        gctx.set_option(B.CM_OPT_EVK_STORED_A, 0)
    assert np.array_equal(gctx.ct_export(sq), gctx.ct_export(gctx.rescale(gctx.relinearize(ref_keys, gctx.mul_ct(x, x)))))
