#!/usr/bin/env python3
"""Benchmark of the homomorphic decode-step VMM on one MI355X.

A step = one pass of the whole hot path over one synthetic input: cm_vmm_pt of an encrypted
4096-vector (interleaved replicated packing) against a plaintext 4096x4096 matrix on the ring
n = 2^16 with 24 ciphertext primes of 50 bits + 4 special primes of 60 bits (6 key-switch
digits), at the top level: 512 plaintext multiply-accumulates, one rescale, and the rotations of
Algorithm 1 — 52 as printed with 32 baby x 16 giant steps (21 full key switches + 31 hoisted); 84 in
the default form, which unrolls the giant steps and the two rotate-and-add ladders into hoisted
rotations, keeps the whole product in the extended basis (one ModDown of both components at the
end) and, its baby steps being cheap, splits 64 x 8.  Keys, weight
plaintexts and the input ciphertext are resident in HBM before the timed region.  --ladders keeps
the ladders, --nested-giants also the nested giant steps, --plain-sums divides every hoisted
rotation by P on its own (Algorithm 1 as printed, 32 x 16, 52 rotations).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--ladders | --nested-giants | --plain-sums]

    python bench.py --workload attention        (config 3, a JSON line of its own; --gqa: every KV head stored once)
    python bench.py --workload prefill          (prompt phase: token-batched product, group append, group attention)
    python bench.py --workload layer            (config 5: one decoder layer's linear path per token on the 36 + 6 ring,
                                                 context 4096 with every KV head stored once, four decode steps)

Prints one JSON line.  `roofline` describes the kernel family with the most time in the step:
achieved = algorithmic bytes per unit / measured time per unit (HIP events around every launch of
the family on its stream), peak = 8 TB/s HBM, traffic = HBM bytes from the committed counter summary under
profiles/ (read from that file, not measured in this run: `traffic_source` names it).
`hbm_probe` = what plain streaming kernels reach on this device (cm_hbm_probe), `frac_of_probe` in every roofline object
the family's rate against the probe of its read/write mix.  `attention_config3` carries the times of configuration 3
(q K^T, scores V and one append against a 1024-token cache; `--workload attention` with and without `--key-index`)
measured in the same run after the timed region (--no-attention leaves them out).
`cpu_baseline` (default --cpu-baseline full): ONE full product of the same workload run by the oracle on the host
cores and timed (Algorithm 1 as printed, 52 rotations, 512 products), plus one key switch on a single thread.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
D = 4096


def measured_traffic():
    """HBM bytes per unit from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE scaled
    by the copy-kernel calibration stated there); keys: 'k_inner_product' (per launch) and
    'ntt_fwd_per_limb'.  Empty if the summary is missing."""
    out = {}
    path = os.path.join(ROOT, "profiles", "pmc_hbm_traffic_bench_config2.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes "):
                _, key, val = line.split()
                out[key.rstrip(":")] = float(val)
    return out


def gpu_setup(raised_sums=True, direct_giants=True, unrolled_ladders=True, stored_a=False):
    import torch
    from paper_2602_11470_amd import binding as B, inputs
    ctx = B.llama_ring(24, 4)
    if stored_a:
        ctx.set_option(B.CM_OPT_EVK_STORED_A, 1)
    x, W = inputs.vmm_inputs(1, D, D)
    plan = ctx.vmm_plan(D, D, W=W, raised_sums=raised_sums, direct_giants=direct_giants,
                        unrolled_ladders=unrolled_ladders)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, plan.steps(), 2)
    t = ctx.S // D
    slots = np.zeros(ctx.S)
    slots[::t] = x
    ct = ctx.encrypt(sk, ctx.encode(slots, ctx.L), 3)
    torch.cuda.synchronize()
    return dict(torch=torch, B=B, ctx=ctx, plan=plan, sk=sk, keys=keys, ct=ct, x=x, W=W, t=t)


def time_steps(g, steps, warmup):
    torch, ctx = g["torch"], g["ctx"]
    y = ctx.vmm_pt(g["keys"], g["plan"], g["ct"])
    for _ in range(warmup):
        ctx.vmm_pt(g["keys"], g["plan"], g["ct"], out=y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.vmm_pt(g["keys"], g["plan"], g["ct"], out=y)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out = ctx.decrypt(g["sk"], y).real[::g["t"]]
    err = float(np.abs(out - g["x"] @ g["W"]).max())
    return dt / steps, err


def kernel_profile(g, steps):
    """The same steps again with every kernel launch bracketed by HIP events on its stream."""
    ctx, B = g["ctx"], g["B"]
    y = ctx.vmm_pt(g["keys"], g["plan"], g["ct"])
    g["torch"].cuda.synchronize()
    ctx.profile_enable(True)
    for _ in range(steps):
        ctx.vmm_pt(g["keys"], g["plan"], g["ct"], out=y)
    g["torch"].cuda.synchronize()
    names = ["ntt_fwd", "ntt_inv", "base_conv", "inner_product", "moddown_finish", "vmm_mac",
             "elementwise", "rescale"]
    fam = {}
    for i, nme in enumerate(names):
        launches, units, ms = ctx.profile_get(i)
        fam[nme] = dict(launches=launches / steps, units=units / steps, ms=ms / steps)
    ctx.profile_enable(False)
    return fam


def time_rotations(g, reps=20):
    """Seconds per un-hoisted rotation, and seconds per launch of its inner-product kernel (k_inner_product, which moves
    the stored key half, the digits and the result of one key switch and shares nothing)."""
    torch, ctx = g["torch"], g["ctx"]
    r = ctx.rotate(g["keys"], g["ct"], 7)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        ctx.rotate(g["keys"], g["ct"], 7, out=r)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / reps
    ctx.profile_enable(True)
    for _ in range(5):
        ctx.rotate(g["keys"], g["ct"], 7, out=r)
    torch.cuda.synchronize()
    launches, _, ms = ctx.profile_get(3)
    ctx.profile_enable(False)
    return sec, ms / launches * 1e-3


def ntt_rates(g, reps=20):
    """Limb transforms per second for batches of 24, 28 and 168 limbs (forward and inverse), timed
    with the library's per-launch HIP events around cm_ntt."""
    torch, ctx = g["torch"], g["ctx"]
    out = {}
    for limbs in (24, 28, 168):
        mods = [i % 28 for i in range(limbs)]
        data = torch.randint(0, 1 << 40, (limbs, ctx.n), dtype=torch.int64, device="cuda")
        for inverse in (False, True):
            for _ in range(2):
                ctx.ntt(data, mods, inverse)
            torch.cuda.synchronize()
            ctx.profile_enable(True)
            for _ in range(reps):
                ctx.ntt(data, mods, inverse)
            torch.cuda.synchronize()
            launches, units, ms = ctx.profile_get(1 if inverse else 0)
            ctx.profile_enable(False)
            out[f"{'inv' if inverse else 'fwd'}_{limbs}"] = units / (ms * 1e-3)
    return out


def calibration_kernel(g):
    """One launch of a plain streaming kernel of known size outside the timed region: the sum of two
    distinct top-level ciphertexts (k_add: reads 2 x 24 MiB, writes 24 MiB).  Counter profiles of
    this script scale FETCH_SIZE / WRITE_SIZE by what they read for this launch."""
    ctx = g["ctx"]
    r = ctx.rotate(g["keys"], g["ct"], 7)
    ctx.add(g["ct"], r)
    g["torch"].cuda.synchronize()


def _oracle_cores():
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def cpu_baseline_sample(raised_sums=True):
    """The oracle's primitives on a bounded sample of the workload (the ring of the benchmark, 3 full rotations,
    one hoisting + 3 hoisted rotations, 8 plaintext multiply-accumulates, one ModDown and one rescale), each timed
    and scaled by the operation counts of Algorithm 1 (21 / 1 / 31 / 512 / 1 / 1): an extrapolation, kept as a
    cross-check of the measured run."""
    from oracle import ckks, params
    prm = params.config2()
    ctx = ckks.Context(prm)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, [7, 64], 2)
    rng = np.random.default_rng(0)
    z = rng.normal(size=ctx.S)
    ct = ctx.encrypt(sk, ctx.encode(z, prm.L), 3)
    w = rng.normal(0, 0.02, ctx.S)

    def timed(fn, reps):
        t0 = time.perf_counter()
        for _ in range(reps):
            r = fn()
        return (time.perf_counter() - t0) / reps, r

    t_hoist, h = timed(lambda: ctx.hoist(ct), 1)
    if raised_sums:
        pt = ctx.encode_ext(w, prm.L)
        t_hrot, R = timed(lambda: ctx.rotate_hoisted_raised(ct, h, 64, keys), 3)
        acc = [np.zeros_like(R[0]), np.zeros_like(R[1])]
        t_mac, _ = timed(lambda: ctx.mac_pt_raised(acc, R, pt, prm.L), 8)
        t_md, x = timed(lambda: ctx.moddown_ct(acc, prm.L, ct.scale * pt.scale), 1)
        t_rot, _ = timed(lambda: ctx.rotate_add_raised(ct, 7, keys, acc), 3)
    else:
        pt = ctx.encode(w, prm.L)
        t_rot, _ = timed(lambda: ctx.rotate(ct, 7, keys), 3)
        t_hrot, _ = timed(lambda: ctx.rotate_hoisted(ct, h, 64, keys), 3)
        x = ctx.mul_pt(ct, pt)
        t_mac, _ = timed(lambda: ctx.mac_pt(x, ct, pt), 8)
        t_md = 0.0
    t_resc, _ = timed(lambda: ctx.rescale(x), 1)
    t_vmm = 21 * t_rot + t_hoist + 31 * t_hrot + 512 * t_mac + t_md + t_resc
    return {"value": 1.0 / t_vmm, "unit": "VMM/s", "cores": _oracle_cores(), "kind": "oracle", "measured": False,
            "sample": "n=2^16, 24+4 primes: 3 rotations, 1 hoisting, 3 hoisted rotations, 8 pt-ct MACs, "
                      + ("1 ModDown, " if raised_sums else "") +
                      "1 rescale timed; scaled by the step's counts 21/1/31/512/" + ("1/" if raised_sums else "") +
                      "1 of Algorithm 1 with its ladders (extrapolated)",
            "key_switch_s": t_rot, "seconds_per_vmm": t_vmm}


_SINGLE_THREAD_KS = r"""
import sys, time
import numpy as np
sys.path.insert(0, sys.argv[1])
from oracle import ckks, params
prm = params.config2()
ctx = ckks.Context(prm)
sk = ctx.keygen_secret(1)
keys = ctx.keygen_rotations(sk, [7], 2)
ct = ctx.encrypt(sk, ctx.encode(np.random.default_rng(0).normal(size=ctx.S), prm.L), 3)
t0 = time.perf_counter()
ctx.rotate(ct, 7, keys)
print(time.perf_counter() - t0)
"""


def cpu_baseline_full():
    """The oracle as it stands, timed on ONE full product of the benchmark's workload (config 2, top level): Algorithm 1
    as printed (preprocess ladder, 31 hoisted baby steps, 512 plaintext products, 15 nested giant steps, reduce ladder,
    rescale: 52 rotations), with the inputs bench.py gives the GPU.  Key generation and encoding are set-up and timed
    apart.  One un-hoisted rotation is also timed on all cores and, in a process of its own with OMP_NUM_THREADS=1, on a
    single thread."""
    import subprocess
    from oracle import ckks, packing, params, vmm
    from paper_2602_11470_amd import inputs
    t_setup = time.perf_counter()
    prm = params.config2()
    ctx = ckks.Context(prm)
    plan = packing.make_plan(ctx.S, D, D)
    x, W = inputs.vmm_inputs(1, D, D)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, plan.all_steps(), 2)
    diags = [[ctx.encode(v, prm.L) for v in row] for row in plan.diagonals(W)]
    ct = ctx.encrypt(sk, ctx.encode(plan.pack_input(x), prm.L), 3)
    t_setup = time.perf_counter() - t_setup
    ctx.rot_count = ctx.ptmul_count = 0
    t0 = time.perf_counter()
    y = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, diags)
    t_vmm = time.perf_counter() - t0
    err = float(np.abs(plan.unpack_output(ctx.decrypt(sk, y).real) - x @ W).max())
    rotations, products = ctx.rot_count, ctx.ptmul_count
    t0 = time.perf_counter()
    ctx.rotate(ct, plan.pre_steps[0], keys)
    t_rot = time.perf_counter() - t0
    env = dict(os.environ, OMP_NUM_THREADS="1")
    t_rot1 = None
    try:
        r = subprocess.run([sys.executable, "-c", _SINGLE_THREAD_KS, ROOT], env=env, capture_output=True, text=True, timeout=300)
        t_rot1 = float(r.stdout.strip().splitlines()[-1])
    except Exception:                                          # reported as missing, never guessed
        pass
    return {"value": 1.0 / t_vmm, "unit": "VMM/s", "cores": _oracle_cores(), "kind": "oracle", "measured": True,
            "sample": "one full 4096x4096 product at config 2 (n=2^16, 24+4 primes, top level), Algorithm 1 as printed: "
                      f"{rotations} rotations, {products} plaintext products, one rescale; oracle.vmm.vmm_pt timed as it stands",
            "seconds_per_vmm": t_vmm, "setup_seconds": t_setup, "max_abs_err_vs_float64": err,
            "key_switch_s": t_rot, "key_switch_s_single_thread": t_rot1}


def attention_workload(a):
    if a.gqa:
        return attention_workload_gqa(a)
    print(json.dumps(attention_result(a)))


def attention_result(a):
    """Config 3 (a line of its own with --workload attention; its times also ride in the default line): one query against an encrypted cache of 1024 tokens, 32 heads
    x 128 dims on the config-2 ring; cache ciphertexts one level below the top.  q K^T = 3 + 128 x
    (relinearisation + 7 rotations) key switches (--ladders); with --shared-dims 1 the 7 rotations unrolled
    into 13 hoisted ones that share 3 ModUps and one ModDown; by default (--shared-dims 128) the copy mask
    applied first, 128 relinearisations and 127 rotations for the whole cache; scores V = 15 hoisted + 7 giant
    + 3 rotations and 8 relinearisations.  Cache contents are random slot vectors (timing does not depend on values;
    parity of this path is in tests/)."""
    import torch
    from paper_2602_11470_amd import binding as B
    ctx = B.llama_ring(24, 4)
    H, E, L = 32, 128, ctx.L
    lv = a.cache_level if a.cache_level > 0 else L - 1
    kv = ctx.kv_create(H, E, lv, r_i=16, unrolled_ladders=not a.ladders, key_index=a.key_index,
                       shared_dims=1 if a.ladders or a.key_index else (a.shared_dims or 128))
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, kv.steps(), 2, with_relin=True)
    rng = np.random.default_rng(3)
    enc = lambda seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), L), seed), lv)
    for c in range(128):
        kv.load(B.CM_QK, c, enc(100 + c))
        kv.load(B.CM_SV, c, enc(300 + c))
        if a.key_index:
            kv.load(B.CM_KV_INDEX, c, enc(500 + c))
    # appends of new tokens (inputs one level above the cache), timed on a nearly full cache
    kv.set_tokens(1024 - 8)
    new_k = ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), L), 20), lv + 1)
    new_v = ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), L), 21), lv + 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(8):
        kv.append(keys, new_k, new_v)
    torch.cuda.synchronize()
    append_ms = (time.perf_counter() - t0) / 8 * 1e3
    assert kv.tokens() == 1024
    q, sc = enc(10), enc(11)
    res = {}
    for name, which, x in (("qk", B.CM_QK, q), ("sv", B.CM_SV, sc)):
        for _ in range(max(1, a.warmup // 2)):
            ctx.vmm_kv(keys, kv, which, x)
        torch.cuda.synchronize()
        reps = max(1, a.steps // 5)
        t0 = time.perf_counter()
        for _ in range(reps):
            ctx.vmm_kv(keys, kv, which, x)
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / reps
    # per key ciphertext: one relinearisation and the sum over the 128 dims, as 7 dependent rotations or,
    # unrolled (runs of 3 + 2 + 2 ladder steps), 13 hoisted ones on 3 ModUps
    sh = 1 if a.ladders or a.key_index else (a.shared_dims or 128)
    per_ct = {1: 13, 2: 14, 4: 10, 8: 6, 16: 7, 32: 3, 64: 1, 128: 0}[sh]    # hoisted rotations of the runs of the ladder left per key ciphertext
    ks_qk = 3 + 15 + 8 + 7 if a.key_index else 3 + 128 * (8 if a.ladders else 1 + per_ct) + sh - 1
    out = {
        "metric": "encrypted-cache attention products/s (config 3: q K^T and scores V, 32 heads x 128 dims, "
                  "context 1024, n=2^16, 24x50-bit + 4x60-bit primes)",
        "value": 1.0 / (res["qk"] + res["sv"]), "unit": "attention steps/s", "n_gpus": 1,
        "higher_is_better": True, "dtype": "u64", "data": "synthetic", "vs_baseline": None,
        "config": {"workload": "config3: q K^T (128 K ciphertexts) + scores V (128 V ciphertexts, 16 baby x 8 giant)",
                   "cache_level": lv,
                   "dim_sum": "none: scores from the key index (15 hoisted rotations of the query, 8 relinearisations, 7 giant steps)"
                              if a.key_index else "rotate-and-add ladder" if a.ladders else
                              "unrolled in the extended basis (3 ModUps, 13 rotations)" if sh == 1 else
                              "mask before the last %d terms: %d rotations per key ciphertext + %d shared" % (sh, per_ct, sh - 1)},
        "qk_ms": res["qk"] * 1e3, "sv_ms": res["sv"] * 1e3, "append_ms": append_ms,
        "qk_key_switches": ks_qk, "qk_key_switches_per_s": ks_qk / res["qk"]}
    del kv, keys, q, sc, new_k, new_v
    ctx.close()
    return out


def attention_workload_gqa(a):
    """Config 3 with every KV head stored once: 8 KV heads x 128 dims, t_kv = 32 tokens per K ciphertext, so the context
    of 1024 tokens is 32 K ciphertexts + 128 V ciphertexts (a quarter of the replicated layout's 128 + 128 at four times
    the capacity); q K^T and scores V run in four passes (inner rotation of the query / of the result, un-replicated
    products).  Same number of ciphertext products as the replicated layout."""
    import torch
    from paper_2602_11470_amd import binding as B
    ctx = B.llama_ring(24, 4)
    Hkv, G, E, L = 8, 4, 128, ctx.L
    lv = a.cache_level if a.cache_level > 0 else L - 2
    kv = ctx.kv_create(Hkv, E, lv, r_i=16, unrolled_ladders=True, key_index=a.key_index,
                       shared_dims=1 if a.key_index else (a.shared_dims or 32))
    gqa = ctx.gqa(kv, G)
    tk = ctx.S // (Hkv * E)
    sk = ctx.keygen_secret(1)
    keys = ctx.keygen_rotations(sk, sorted({s_ for s_ in kv.steps() if s_ % tk == 0} | set(gqa.steps())), 2, with_relin=True)
    rng = np.random.default_rng(3)
    enc = lambda seed, level: ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), L), seed), level)
    nk = 1024 // tk
    for c in range(nk):
        kv.load(B.CM_QK, c, enc(100 + c, lv))
    for c in range(E):
        kv.load(B.CM_SV, c, enc(300 + c, lv))
        if a.key_index:
            kv.load(B.CM_KV_INDEX, c, enc(500 + c, lv))
    kv.set_tokens(1024 - 8)
    new_k, new_v = enc(20, lv + 1), enc(21, lv + 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(8):
        kv.append(keys, new_k, new_v)
    torch.cuda.synchronize()
    append_ms = (time.perf_counter() - t0) / 8 * 1e3
    q = enc(10, lv + 1)
    scores = [enc(11 + d, lv) for d in range(G)]
    res = {}
    for name, fn in (("qk", lambda: ctx.gqa_qk(keys, gqa, q)), ("sv", lambda: ctx.gqa_sv(keys, gqa, scores))):
        for _ in range(max(1, a.warmup // 2)):
            fn()
        torch.cuda.synchronize()
        reps = max(1, a.steps // 5)
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / reps
    free, total = torch.cuda.mem_get_info()
    print(json.dumps({
        "metric": "encrypted-cache attention products/s (config 3: q K^T and scores V, 32 query heads on 8 KV heads x 128 dims, "
                  "context 1024, n=2^16, 24x50-bit + 4x60-bit primes; every KV head stored once)",
        "value": 1.0 / (res["qk"] + res["sv"]), "unit": "attention steps/s", "n_gpus": 1,
        "higher_is_better": True, "dtype": "u64", "data": "synthetic", "vs_baseline": None,
        "config": {"workload": "config3, GQA-native: q K^T (32 K ciphertexts x 4 passes) + scores V (128 V ciphertexts x 4 passes)",
                   "cache_level": lv, "shared_dims": 1 if a.key_index else (a.shared_dims or 32), "key_index": bool(a.key_index),
                   "cache_ciphertexts": nk + E * (2 if a.key_index else 1)},
        "qk_ms": res["qk"] * 1e3, "sv_ms": res["sv"] * 1e3, "append_ms": append_ms,
        "device_bytes_in_use": total - free}))


def layer_workload(a):
    """Config 5: the linear path of one Llama-3-8B-shaped decoder layer per token on the ring of 36 + 6 primes, context
    4096 in ONE cache that stores the 8 KV heads once (128 K + 128 V ciphertexts), four decode steps: q projection
    (4096 x 4096), k / v projections (4096 x 1024, one shared-baby-step call, outputs on the residue of the token), rotary
    embedding of q and k, append, q K^T and scores V in four passes each, extraction, output projection, gate / up (one
    call) and down.  Where the model has a non-linear layer (softmax, normalisation, SiLU) the next stage starts from a
    resident ciphertext at the level the stage runs at.  Everything is resident in HBM before the timed region."""
    import torch
    from paper_2602_11470_amd import binding as B
    t_setup = time.perf_counter()
    ctx = B.llama_ring(36, 6)
    H, Hkv, G, E, d, dm, L = 32, 8, 4, 128, 4096, 16384, ctx.L
    t, tk = ctx.S // d, ctx.S // (Hkv * E)
    cache_lv = L - 3                       # projection, rotary embedding, append mask: one level each
    o_lv = cache_lv - 3                    # scores V (one level), the move back to the query heads' runs, the extraction
    mlp_lv, down_lv = 12, 10               # the MLP further down the chain (the paper runs it at its lowest levels, Table 5)
    rng = np.random.default_rng(5)
    Wsq = lambda: rng.normal(0, 0.02, (d, d))
    sk = ctx.keygen_secret(1)
    index = not a.no_key_index
    kv = ctx.kv_create(Hkv, E, cache_lv, r_i=16, unrolled_ladders=True, key_index=index,
                       shared_dims=1 if index else (a.shared_dims or 128))
    gqa = ctx.gqa(kv, G)
    plan_q = ctx.vmm_plan(d, d, W=Wsq(), level=L, unrolled_ladders=True)
    plan_o = ctx.vmm_plan(d, d, W=Wsq(), level=o_lv, unrolled_ladders=True)
    plan_g = ctx.vmm_plan(d, dm, W=rng.normal(0, 0.02, (d, dm)), level=mlp_lv, unrolled_ladders=True)
    plan_u = ctx.vmm_plan(d, dm, W=rng.normal(0, 0.02, (d, dm)), level=mlp_lv, unrolled_ladders=True)
    plan_d = ctx.vmm_plan(dm, d, W=rng.normal(0, 0.02, (dm, d)), level=down_lv, unrolled_ladders=True)
    n0 = 4096 - 4
    taus = [(n0 + i) % tk for i in range(4)]
    Wk, Wv = rng.normal(0, 0.02, (d, Hkv * E)), rng.normal(0, 0.02, (d, Hkv * E))
    plans_kv = [(ctx.vmm_plan(d, Hkv * E, W=Wk, level=L, tau=tau, unrolled_ladders=True),
                 ctx.vmm_plan(d, Hkv * E, W=Wv, level=L, tau=tau, unrolled_ladders=True)) for tau in taus]
    ropes_q = [ctx.rope(H, E, L - 1, n0 + i, 0) for i in range(4)]
    ropes_k = [ctx.rope(Hkv, E, L - 1, n0 + i, taus[i]) for i in range(4)]
    steps = {s_ for s_ in kv.steps() if s_ % tk == 0} | set(gqa.steps()) | {H * t, -H * t, Hkv * tk, -Hkv * tk}
    for p in [plan_q, plan_o, plan_g, plan_u, plan_d] + [p for pair in plans_kv for p in pair]:
        steps |= set(p.steps())
    keys = ctx.keygen_rotations(sk, sorted(steps), 2, with_relin=True)
    enc = lambda level, seed, scale=0.0: ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), L, scale), seed), level)
    mods = ctx.moduli()
    proj_scale = ctx.scale * ctx.scale / float(mods[L])          # a cache holds one scale: the one a projection leaves
    for c in range(128):
        kv.load(B.CM_QK, c, enc(cache_lv, 100 + c, proj_scale))
        kv.load(B.CM_SV, c, enc(cache_lv, 300 + c, proj_scale))
        if index:
            kv.load(B.CM_KV_INDEX, c, enc(cache_lv, 500 + c, proj_scale))
    residue0 = np.zeros(ctx.S)
    residue0[::t] = 1.0
    mask = ctx.encode(residue0, cache_lv - 2, float(mods[cache_lv - 2]), mont=True)
    x = enc(L, 500)
    scores = [enc(cache_lv, 700 + d_) for d_ in range(G)]
    h_in, act = enc(mlp_lv, 800), enc(down_lv, 900)
    torch.cuda.synchronize()
    free, total = torch.cuda.mem_get_info()
    t_setup = time.perf_counter() - t_setup

    def run():
        kv.set_tokens(n0)
        marks = []
        for i in range(4):
            e0 = torch.cuda.Event(enable_timing=True)
            e0.record()
            gq = ctx.vmm_pt(keys, plan_q, x)
            gk, gv = ctx.vmm_pt_multi(keys, list(plans_kv[i]), x)
            gq = ctx.rope_apply(keys, ropes_q[i], gq)
            gk = ctx.rope_apply(keys, ropes_k[i], gk)
            kv.append(keys, gk, ctx.level_drop(gv, L - 2))
            e1 = torch.cuda.Event(enable_timing=True)
            e1.record()
            ctx.gqa_qk(keys, gqa, gq)
            e2 = torch.cuda.Event(enable_timing=True)
            e2.record()
            ga = ctx.gqa_sv(keys, gqa, scores)
            e3 = torch.cuda.Event(enable_timing=True)
            e3.record()
            ctx.vmm_pt(keys, plan_o, ctx.rescale(ctx.mul_pt(ga, mask)))
            ctx.vmm_pt_multi(keys, [plan_g, plan_u], h_in)
            ctx.vmm_pt(keys, plan_d, act)
            e4 = torch.cuda.Event(enable_timing=True)
            e4.record()
            marks.append((e0, e1, e2, e3, e4))
        torch.cuda.synchronize()
        return marks

    run()                                   # warm-up: per-level tables, allocator
    t0 = time.perf_counter()
    marks = run()
    sec = (time.perf_counter() - t0) / 4
    parts = np.array([[m[j].elapsed_time(m[j + 1]) for j in range(4)] for m in marks]).mean(axis=0)
    print(json.dumps({
        "metric": "decoder-layer linear path per token (config 5: n=2^16, 36x50-bit + 6x60-bit primes, dnum 6; context 4096, "
                  "8 KV heads stored once; four decode steps)",
        "value": 1.0 / sec, "unit": "decode steps/s", "ms_per_step": sec * 1e3, "n_gpus": 1, "steps": 4,
        "higher_is_better": True, "dtype": "u64", "data": "synthetic", "vs_baseline": None,
        "config": {"workload": "config5: q, k, v, o, gate, up, down projections + rotary embedding + append + q K^T + scores V "
                               "per token, context 4096",
                   "levels": {"input": L, "cache": cache_lv, "output_projection": o_lv, "gate_up": mlp_lv, "down": down_lv},
                   "rotation_keys": len(steps), "cache_ciphertexts": 384 if index else 256,
                   "q_k_transposed": "from the key index (the scores V schedule per pass)" if index else
                                     "copy mask in front of the sum over the dims, %d shared rotations per pass" % ((a.shared_dims or 128) - 1)},
        "ms": {"projections_rope_append": float(parts[0]), "qk": float(parts[1]), "sv": float(parts[2]),
               "o_gate_up_down": float(parts[3])},
        "device_bytes_resident": int(total - free), "setup_seconds": t_setup}))


def sweep_workload(a):
    """Square projections of the paper's three model widths (Table 4) and its level sweep, in the
    default form (raised sums, unrolled giant steps): ms per product.  A JSON line of its own."""
    import torch
    from paper_2602_11470_amd import binding as B, inputs
    ctx = B.llama_ring(24, 4)
    sk = ctx.keygen_secret(1)
    rows = []
    shapes = ((4096, 4096, 23), (4096, 4096, 13), (4096, 4096, 4), (4096, 4096, 1), (2048, 2048, 23), (1024, 1024, 23),
              (4096, 16384, 23), (16384, 4096, 23))          # the last two: MLP up / down (14336 padded to 16384)
    for d_in, d_out, level in shapes:
        x, W = inputs.vmm_inputs(1, d_in, d_out)
        plan = ctx.vmm_plan(d_in, d_out, W=W, level=level, unrolled_ladders=True)
        keys = ctx.keygen_rotations(sk, plan.steps(), 2)
        d = min(d_in, d_out)
        t, tp = ctx.S // d, ctx.S // max(d_in, d_out)
        slots = np.zeros(ctx.S)
        if d_in <= d_out:
            slots[::t] = x                                       # x[b] at slot b t
        else:
            for s_ in range(d_in // d):
                slots[s_ * tp::t] = x[s_ * d:(s_ + 1) * d]       # x[b + s d] at slot b t + s t'
        ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(slots, ctx.L), 3), level)
        y = ctx.vmm_pt(keys, plan, ct)
        for _ in range(a.warmup):
            ctx.vmm_pt(keys, plan, ct, out=y)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            ctx.vmm_pt(keys, plan, ct, out=y)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / a.steps * 1e3
        out = ctx.decrypt(sk, y).real
        ref = x @ W
        if d_out <= d_in:
            got = out[::t]                                       # y[c] at slot c t
        else:
            got = np.concatenate([out[s_ * tp::t] for s_ in range(d_out // d)])   # y[b + s d] at b t + s t'
        err = float(np.abs(got - ref).max())
        rows.append({"d_in": d_in, "d_out": d_out, "level": level, "rotations": plan.n_rotations, "pt_mults": plan.r_i * plan.r_o,
                     "ms": ms, "max_abs_err": err})
        del plan, keys
    # the q / k / v projections of one token: one input, three weight matrices of one shape; the
    # preprocess rotations and the hoisted baby steps run once (cm_vmm_pt_multi)
    d, level = 4096, ctx.L
    x, _ = inputs.vmm_inputs(1, d, d)
    plans = [ctx.vmm_plan(d, d, W=inputs.vmm_inputs(2 + i, d, d)[1], level=level, unrolled_ladders=True) for i in range(3)]
    keys = ctx.keygen_rotations(sk, plans[0].steps(), 2)
    slots = np.zeros(ctx.S)
    slots[::ctx.S // d] = x
    ct = ctx.encrypt(sk, ctx.encode(slots, ctx.L), 3)
    outs = ctx.vmm_pt_multi(keys, plans, ct)
    qkv = {}
    for name, fn in (("three single products", lambda: [ctx.vmm_pt(keys, p, ct, out=o) for p, o in zip(plans, outs)]),
                     ("one shared-baby-step call", lambda: ctx.vmm_pt_multi(keys, plans, ct, outs))):
        for _ in range(a.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            fn()
        torch.cuda.synchronize()
        qkv[name] = (time.perf_counter() - t0) / a.steps * 1e3
    print(json.dumps({"metric": "ms per homomorphic VMM, widths of Table 4 and levels 23/13/4/1 (n=2^16, 24+4 primes)",
                      "unit": "ms", "n_gpus": 1, "data": "synthetic", "dtype": "u64", "rows": rows,
                      "qkv_projections_ms": qkv}))


def prefill_workload(a):
    """The prompt phase (Sec. 5.4) on the config-2 ring: one 4096 x 4096 product over a ciphertext of
    t = 8 tokens (4096 diagonals as 128 baby x 32 giant steps, 158 rotations), the rotary embedding of a
    token group and the append of a token group to the 32 x 128 cache.  A JSON line of its own."""
    import torch
    from paper_2602_11470_amd import binding as B
    ctx = B.llama_ring(24, 4)
    sk = ctx.keygen_secret(1)
    d, t = 4096, ctx.S // 4096
    rng = np.random.default_rng(5)
    X, W = rng.uniform(-1, 1, size=(t, d)), rng.uniform(-1, 1, size=(d, d)) / 64

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    rows = []
    for level in (ctx.L, 4):
        plan = ctx.vmm_plan(d, d, W=W, level=level, direct_giants=True, token_batch=True)
        keys = ctx.keygen_rotations(sk, plan.steps(), 2)
        ct = ctx.level_drop(ctx.encrypt(sk, ctx.encode(X.T.reshape(-1), ctx.L), 3), level)   # X[tau, b] at b t + tau
        y = ctx.vmm_pt(keys, plan, ct)
        ms = timed(lambda: ctx.vmm_pt(keys, plan, ct, out=y), max(2, a.steps // 4))
        err = float(np.abs(ctx.decrypt(sk, y).real.reshape(d, t).T - X @ W).max())
        rows.append({"level": level, "tokens_per_ciphertext": t, "rotations": plan.n_rotations, "pt_mults": plan.r_i * plan.r_o,
                     "ms": ms, "ms_per_token": ms / t, "max_abs_err": err})
        del plan, keys
    H, E, lv = 32, 128, ctx.L - 3
    kv = ctx.kv_create(H, E, lv, r_i=16)
    rope = ctx.rope(H, E, lv + 2, 0, tau=-1)
    keys = ctx.keygen_rotations(sk, sorted(set(kv.steps()) | set(rope.steps())), 2, with_relin=True)
    kg = ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), ctx.L), 20), lv + 2)
    vg = ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), ctx.L), 21), lv + 1)
    kr = ctx.rope_apply(keys, rope, kg)
    rope_ms = timed(lambda: ctx.rope_apply(keys, rope, kg, out=kr), a.steps)

    irot = ctx.inner_rot(ctx.S // (H * E), 3, lv + 2)
    ikeys = ctx.keygen_rotations(sk, irot.steps(), 2)
    qi = ctx.rope_apply(ikeys, irot, kg)
    inner_ms = timed(lambda: ctx.rope_apply(ikeys, irot, kg, out=qi), a.steps)

    def append():
        kv.set_tokens(0)
        kv.append_group(keys, kr, vg)
    append_ms = timed(append, a.steps)
    del kv, keys
    # attention of a query group against a prompt of 128 tokens (16 K ciphertexts, all 128 V ciphertexts), for one
    # delta: q K^T without replication, scores V without the sum over the residues; a group takes t of each plus
    # 2 (t - 1) inner rotations
    tk = ctx.S // (H * E)
    kva = ctx.kv_create(H, E, lv, r_i=16, unrolled_ladders=True, key_index=a.key_index,
                        shared_dims=1 if a.key_index else (a.shared_dims or 16))
    akeys = ctx.keygen_rotations(sk, [s_ for s_ in kva.steps() if s_ % tk == 0], 2, with_relin=True)
    encl = lambda seed: ctx.level_drop(ctx.encrypt(sk, ctx.encode(rng.normal(size=ctx.S), ctx.L), seed), lv)
    for c in range(128):
        if c < 16:
            kva.load(B.CM_QK, c, encl(100 + c))
        kva.load(B.CM_SV, c, encl(300 + c))
        if a.key_index:
            kva.load(B.CM_KV_INDEX, c, encl(500 + c))
    kva.set_tokens(16 * tk)
    qg, sg = encl(10), encl(11)
    qk_ms = timed(lambda: ctx.vmm_kv(akeys, kva, B.CM_QK_GROUP, qg), max(2, a.steps // 4))
    sv_ms = timed(lambda: ctx.vmm_kv(akeys, kva, B.CM_SV_GROUP, sg), max(2, a.steps // 4))
    print(json.dumps({"metric": "prompt phase, ms per ciphertext of 8 tokens (n=2^16, 24+4 primes)", "unit": "ms", "n_gpus": 1,
                      "data": "synthetic", "dtype": "u64", "token_batched_4096x4096": rows,
                      "rope_group_ms": rope_ms, "inner_rotation_ms": inner_ms, "append_group_ms": append_ms,
                      "append_group_ms_per_token": append_ms / tk,
                      "group_attention_prompt_128": {"cache_level": lv, "shared_dims": 1 if a.key_index else (a.shared_dims or 16), "key_index": bool(a.key_index),
                                                     "qk_group_ms_per_delta": qk_ms,
                                                     "sv_group_ms_per_delta": sv_ms,
                                                     "ms_per_group": tk * (qk_ms + sv_ms) + 2 * (tk - 1) * inner_ms}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="same as --cpu-baseline none")
    ap.add_argument("--cpu-baseline", choices=["full", "sample", "none"], default="full",
                    help="full (default): one full product of the workload timed on the oracle (about two minutes of host "
                         "time) and the extrapolation from a sample beside it; sample: the extrapolation only; none")
    ap.add_argument("--no-attention", action="store_true", help="leave the configuration-3 attention times out of the default line")
    ap.add_argument("--stored-a", action="store_true",
                    help="evaluation keys with both halves in device memory (CM_OPT_EVK_STORED_A): the inner products read the "
                         "uniform half instead of regenerating it")
    ap.add_argument("--no-key-index", action="store_true",
                    help="layer workload: q K^T from the K cache itself instead of the key index")
    ap.add_argument("--gqa", action="store_true",
                    help="attention workload: the cache stores the 8 KV heads once (32 K ciphertexts of 32 tokens), q K^T and "
                         "scores V run in four passes (cm_gqa_*)")
    ap.add_argument("--shared-dims", type=int, default=0,
                    help="attention / prefill workloads: terms of the sum over the dims of q K^T taken after the copy mask, by "
                         "rotations shared by all key ciphertexts (1 = the printed order; default 128 for the 128 key "
                         "ciphertexts of the attention workload, 16 for the 16 of the prefill workload)")
    ap.add_argument("--key-index", action="store_true",
                    help="attention / prefill workloads: the cache also keeps the key index (a diagonal re-layout of the K cache maintained "
                         "at append); q K^T runs on it like scores V")
    ap.add_argument("--ladders", action="store_true",
                    help="preprocess and reduce as the rotate-and-add ladders of Algorithm 1 (3 + 3 dependent rotations)")
    ap.add_argument("--nested-giants", action="store_true",
                    help="giant steps in the nested (Horner) form with one key, as Algorithm 1 prints them")
    ap.add_argument("--plain-sums", action="store_true",
                    help="divide every hoisted rotation by P on its own (31 more ModDowns per step)")
    ap.add_argument("--cache-level", type=int, default=0, help="attention workload: level of the cache (default L-1)")
    ap.add_argument("--workload", choices=["projection", "attention", "sweep", "prefill", "layer"], default="projection",
                    help="projection = config 2 (the benchmark line); attention = config 3; sweep = other widths "
                         "and levels; the last two print a line of their own")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if a.workload == "attention":
        attention_workload(a)
        return
    if a.workload == "prefill":
        prefill_workload(a)
        return
    if a.workload == "sweep":
        sweep_workload(a)
        return
    if a.workload == "layer":
        layer_workload(a)
        return
    nested = a.plain_sums or a.nested_giants
    g = gpu_setup(raised_sums=not a.plain_sums, direct_giants=not nested, unrolled_ladders=not (nested or a.ladders),
                  stored_a=a.stored_a)
    sec, err = time_steps(g, a.steps, a.warmup)
    if not err < 1e-4:
        print(f"bench.py: decrypted result off by {err}", file=sys.stderr)
        sys.exit(1)
    fam = kernel_profile(g, min(a.steps, 5))
    t_rot, t_ip_single = time_rotations(g)
    calibration_kernel(g)
    rates = ntt_rates(g)
    n, limbs, K, beta = g["ctx"].n, 24, 4, 6
    limb_bytes = 8 * n
    # dominant kernel family of the step by time
    dom = max(fam, key=lambda k: fam[k]["ms"])
    ntt = fam["ntt_fwd"]
    ntt_per_launch_limbs = ntt["units"] / ntt["launches"]
    ntt_launch_s = ntt["ms"] / ntt["launches"] * 1e-3
    # forward NTT: algorithmic bytes = read + write each limb once (1 MiB per 2^16-point limb)
    ntt_gbs = ntt_per_launch_limbs * 2 * limb_bytes / ntt_launch_s / 1e9
    # inner products: a launch of the batched kernel carries several (63 hoisted rotations, 7 giant
    # steps), so the figure is per inner product: family time / inner products
    ip = fam["inner_product"]
    ip_launch_s = ip["ms"] / ip["units"] * 1e-3
    ext = limbs + K
    # Algorithmic bytes of the family per step.  W = one polynomial on the extended basis; an inner product on its own
    # moves the stored half of its key (the uniform half is regenerated from its seed in the kernel), the raised digits
    # and the two-component result.  In the default form the launches share operands: the baby steps read the digits
    # and the first component once for all keys; the giant steps and each ladder run write one sum.
    W_ = limb_bytes * ext
    kh = 2 if a.stored_a else 1                                                      # key halves read from HBM
    plan = g["plan"]
    default_form = not (nested or a.ladders)
    if default_form:
        runs = 2 * -(-int(np.log2(g["t"])) // 3)                                  # preprocess and reduce ladders, runs of <= 3 steps
        ladder_amounts = plan.n_rotations - (plan.r_i - 1) - (plan.r_o - 1)
        ip_family_bytes = ((beta * W_ + W_) + (plan.r_i - 1) * (kh * beta * W_ + 2 * W_)            # baby steps
                           + (plan.r_o - 1) * ((1 + kh) * beta * W_ + W_) + 4 * W_                # giant steps into one sum
                           + runs * (beta * W_ + W_ + 4 * W_) + ladder_amounts * kh * beta * W_)  # ladder runs
    else:
        ip_family_bytes = ip["units"] * ((1 + kh) * beta * W_ + 2 * W_)    # every inner product on its own
    ip_bytes = ip_family_bytes / ip["units"]                                      # per inner product, on average
    ip_gbs = ip_bytes / ip_launch_s / 1e9
    mac = fam["vmm_mac"]
    mac_bytes = limb_bytes * ext * (plan.r_i * plan.r_o + 2 * plan.r_i + 2 * plan.r_o) if not a.plain_sums else \
        limb_bytes * limbs * (plan.r_i * plan.r_o + 2 * plan.r_i + 2 * plan.r_o)
    mac_s = mac["ms"] / mac["launches"] * 1e-3
    mac_gbs = mac_bytes / mac_s / 1e9
    tr = measured_traffic()
    ntt_traffic = tr["ntt_fwd_per_limb"] * ntt_per_launch_limbs if "ntt_fwd_per_limb" in tr else None
    roofs = {
        "ntt_fwd": {"bound": "hbm", "achieved": ntt_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ntt_gbs / HBM_PEAK_GBS, "traffic": ntt_traffic,
                    "kernel": "ntt_cols_fwd+ntt_rows256_fwd (one launch of the pair)",
                    "limbs_per_launch": ntt_per_launch_limbs, "us_per_launch": ntt_launch_s * 1e6},
        "inner_product": {"bound": "hbm", "achieved": ip_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": ip_gbs / HBM_PEAK_GBS,
                          "traffic": (tr["inner_product_family_per_step"] / ip["units"]
                                      if default_form and "inner_product_family_per_step" in tr else None),
                          "kernel": "k_inner_product_fanout (the hoisted baby steps, digits read once per 8 keys) + "
                                    "k_inner_product_batch (giant steps, ladder runs): per inner product, averaged over "
                                    "the inner products of a step",
                          "algorithmic_bytes_per_inner_product": ip_bytes,
                          "inner_products_per_step": ip["units"], "launches_per_step": ip["launches"],
                          "us_per_launch": ip_launch_s * 1e6},
        "inner_product_single": {"bound": "hbm", "achieved": ((1 + kh) * beta * W_ + 2 * W_) / t_ip_single / 1e9, "peak": HBM_PEAK_GBS,
                                 "unit": "GB/s", "frac": ((1 + kh) * beta * W_ + 2 * W_) / t_ip_single / 1e9 / HBM_PEAK_GBS,
                                 "traffic": tr.get("k_inner_product"),
                                 "kernel": "k_inner_product (the inner product of one un-hoisted key switch)",
                                 "us_per_launch": t_ip_single * 1e6},
        "vmm_mac": {"bound": "hbm", "achieved": mac_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": mac_gbs / HBM_PEAK_GBS,
                    "traffic": tr.get("k_vmm_mac_lds"), "kernel": "k_vmm_mac_lds (one launch per step)",
                    "algorithmic_bytes_per_launch": mac_bytes, "us_per_launch": mac_s * 1e6},
    }
    # What plain streaming kernels of the same read/write mix reach on this device (cm_hbm_probe), and each family's rate
    # as a fraction of it.  The transform pair moves every limb twice in each direction (column pass, row pass), so its
    # traffic is twice its algorithmic bytes.
    B = g["B"]
    probe = {"read": B.hbm_probe(B.CM_PROBE_READ), "read1_write1": B.hbm_probe(B.CM_PROBE_COPY),
             "read3_write1": B.hbm_probe(B.CM_PROBE_READ3_WRITE1), "unit": "GB/s",
             "what": "best of 5 passes of a plain streaming kernel over 4 GiB (16-byte non-temporal accesses): reads only; one "
                     "read and one write stream; three read streams and one write stream"}
    roofs["ntt_fwd"]["frac_of_probe"] = 2 * ntt_gbs / probe["read1_write1"]
    roofs["ntt_fwd"]["probe"] = "read1_write1, against the pair's traffic of 2 MiB per limb"
    roofs["inner_product"]["frac_of_probe"] = ip_gbs / probe["read3_write1"]
    roofs["inner_product"]["probe"] = "read3_write1"
    roofs["inner_product_single"]["frac_of_probe"] = roofs["inner_product_single"]["achieved"] / probe["read"]
    roofs["inner_product_single"]["probe"] = "read (15 words read per word written)"
    roofs["vmm_mac"]["frac_of_probe"] = mac_gbs / probe["read"]
    roofs["vmm_mac"]["probe"] = "read"
    roofline = roofs.get(dom, roofs["inner_product"])
    ks_bytes = limb_bytes * (kh * beta * ext + limbs + 2 * limbs)        # stored key halves once + input + output
    out = {
        "metric": "homomorphic VMMs/s (d=4096 projection, n=2^16, 24x50-bit + 4x60-bit primes, top level)",
        "value": 1.0 / sec, "unit": "VMM/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": "config2: encrypted 4096-vector x plaintext 4096x4096, interleaved replicated "
                               f"packing, BSGS {g['plan'].r_i}x{g['plan'].r_o}, {g['plan'].n_rotations} rotations, 512 pt-ct MACs",
                   "ring_degree": n,
                   "baby_step_sums": "plain" if a.plain_sums else "extended basis",
                   "giant_steps": "nested (one key)" if nested else "unrolled (one key per step)",
                   "ladders": "rotate-and-add, 3 + 3 dependent rotations" if (nested or a.ladders) else
                              "unrolled: 7 + 7 hoisted rotations, whole product in the extended basis",
                   "rotation_keys": len(set(g["plan"].steps())),
                   "key_halves_in_hbm": kh,
                   "ciphertext_primes": limbs, "special_primes": K, "dnum": beta, "level": limbs - 1},
        "max_abs_err_vs_float64": err,
        "key_switches_per_s": 1.0 / t_rot, "key_switch_us": t_rot * 1e6,
        "key_switch_algorithmic_gbs": ks_bytes / t_rot / 1e9,
        "key_switch_frac_of_hbm_peak": ks_bytes / t_rot / 1e9 / HBM_PEAK_GBS,
        "limb_ntts_per_s": ntt["units"] / (ntt["ms"] * 1e-3),
        "limb_ntts_per_s_by_batch": {k: round(v) for k, v in rates.items()},
        "kernel_ms_per_step": {k: round(v["ms"], 4) for k, v in fam.items()},
        "dominant_kernel_family": dom,
        "roofline": roofline,
        "hbm_probe": probe,
        "traffic_source": "profiles/pmc_hbm_traffic_bench_config2.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary committed "
                          "with the code, which names the commit it measured; read from the file, not measured in this run)",
        "roofline_inner_product": roofs["inner_product"],
        "roofline_vmm_mac": roofs["vmm_mac"],
        "roofline_key_switch_inner_product": roofs["inner_product_single"],
        "roofline_ntt_fwd": roofs["ntt_fwd"],
    }
    g.clear()                                            # keys, plaintexts and context of the product go back
    if not a.no_attention:
        # configuration 3 beside the headline: one query against the 1024-token cache of 32 heads x 128 dims at level 22,
        # in the workload's default form and with the key index (what `--workload attention [--key-index]` prints)
        import copy
        att = {}
        for name, ki in (("copy_mask_first", False), ("key_index", True)):
            b = copy.copy(a)
            b.gqa, b.key_index, b.ladders, b.shared_dims, b.cache_level = False, ki, False, 0, 0
            r = attention_result(b)
            att[name] = {k: round(r[k], 3) for k in ("qk_ms", "sv_ms", "append_ms")}
        out["attention_config3"] = att
    mode = "none" if a.no_cpu_baseline else a.cpu_baseline
    if mode != "none":
        g.clear()                                        # the GPU's memory and the host's cores go back before the oracle runs
        sample = cpu_baseline_sample(raised_sums=not a.plain_sums)
        if mode == "full":
            out["cpu_baseline"] = cpu_baseline_full()
            out["cpu_baseline"]["extrapolated_seconds_per_vmm"] = sample["seconds_per_vmm"]
        else:
            out["cpu_baseline"] = sample
    print(json.dumps(out))


if __name__ == "__main__":
    main()
