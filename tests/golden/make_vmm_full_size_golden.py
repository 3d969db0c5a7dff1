"""Writes tests/golden/vmm_full_size.txt (with the argument `raised`: vmm_full_size_raised.txt; with
`direct`: vmm_full_size_direct.txt; with `unrolled`: vmm_full_size_unrolled.txt) by running ONLY the oracle.

Full-size parity case of the packed product: ring n = 2^16 with 24 x 50-bit + 4 x 60-bit primes
(benchmark configuration 2), d = 4096 square plan (32 baby x 16 giant steps, 52 rotations, 512
plaintext multiply-accumulates), top level.  Plaintexts enter as integer coefficient polynomials
drawn from a seeded integer generator (ciphertext-level parity does not care what they encode,
and integers cross between machines bit for bit, which encoded floats need not).

The fixture stores a SHA-256 of the canonical output ciphertext and the first coefficients of
every limb.  Run from the repository root:
    python tests/golden/make_vmm_full_size_golden.py            (Algorithm 1 as printed)
    python tests/golden/make_vmm_full_size_golden.py raised     (baby-step sums kept in the extended basis)
    python tests/golden/make_vmm_full_size_golden.py direct     (that, with the giant steps unrolled)
    python tests/golden/make_vmm_full_size_golden.py unrolled   (that, with the two ladders unrolled too, 64 x 8 steps: 84 rotations)
    python tests/golden/make_vmm_full_size_golden.py mlp_up     (vmm_full_size_mlp_up.txt: 4096 -> 16384, the MLP up / gate shape with
                                                                 14336 padded to 16384 (App. C, non-square), unrolled form, 128 x 16
                                                                 steps, 2048 products, at the paper's operating level 4)
    python tests/golden/make_vmm_full_size_golden.py mlp_down   (vmm_full_size_mlp_down.txt: 16384 -> 4096, the same for the down projection)
(a few minutes each on 8 cores, ~20 GiB of memory).
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ckks, packing, params, vmm  # noqa: E402

SEED_X, SEED_W, SEED_SK, SEED_EVK, SEED_ENC = 11, 12, 1, 2, 3
D = 4096


def integer_inputs(n, plan):
    """x plaintext: uniform integers below 2^48 in magnitude; diagonal (j, k): below 2^44."""
    xc = np.random.default_rng(SEED_X).integers(-2 ** 48, 2 ** 48, n, dtype=np.int64)
    rng = np.random.default_rng(SEED_W)
    diag = [rng.integers(-2 ** 44, 2 ** 44, n, dtype=np.int64) for _ in range(plan.r_i * plan.r_o)]
    return xc, diag


MLP_WIDE, MLP_LEVEL = 16384, 4


def plan_for(S, form):
    """32 baby x 16 giant steps (the 52 rotations of Table 2); the unrolled form, which is the one bench.py
    times, with the split it runs there: 64 x 8.  The MLP shapes (2048 diagonals) with the split the library
    takes for them in the unrolled form: 128 x 16."""
    if form == "mlp_up":
        return packing.make_plan(S, D, MLP_WIDE, r_i=128)
    if form == "mlp_down":
        return packing.make_plan(S, MLP_WIDE, D, r_i=128)
    return packing.make_plan(S, D, D, r_i=64 if form == "unrolled" else None)


def level_for(prm, form):
    return MLP_LEVEL if form.startswith("mlp") else prm.L


def main(form="plain"):
    mlp = form.startswith("mlp")
    raised, direct, unrolled = form in ("raised", "direct", "unrolled") or mlp, form == "direct", form == "unrolled" or mlp
    t0 = time.time()
    prm = params.config2()
    ctx = ckks.Context(prm)
    level = level_for(prm, form)
    plan = plan_for(ctx.S, form)
    xc, diag = integer_inputs(ctx.n, plan)
    sk = ctx.keygen_secret(SEED_SK)
    steps = vmm.unrolled_steps(plan) if unrolled else vmm.direct_giant_steps(plan) if direct else plan.all_steps()
    keys = ctx.keygen_rotations(sk, steps, SEED_EVK)
    print("keys", len(keys), time.time() - t0, flush=True)
    ct = ctx.level_drop(ctx.encrypt(sk, ctx.pt_from_coeffs(xc, prm.L, prm.scale), SEED_ENC), level)
    make_pt = ctx.pt_from_coeffs_ext if raised else ctx.pt_from_coeffs
    pts = [[make_pt(diag[j * plan.r_o + k], level, prm.scale) for k in range(plan.r_o)] for j in range(plan.r_i)]
    print("plaintexts", time.time() - t0, flush=True)
    if unrolled:
        y = vmm.vmm_pt_unrolled(ctx, keys, plan, ct, pts)
    elif direct:
        y = vmm.vmm_pt_direct_giants(ctx, keys, plan, ct, pts)
    elif raised:
        y = vmm.vmm_pt_double_hoisted(ctx, keys, plan, ct, pts)
    else:
        y = vmm.vmm_pt(vmm.CkksOps(ctx, keys), plan, ct, pts)
    can = ctx.canonical(y)
    print("vmm", time.time() - t0, ctx.rot_count, ctx.ptmul_count, flush=True)
    out = os.path.join(ROOT, "tests", "golden", {"plain": "vmm_full_size.txt", "raised": "vmm_full_size_raised.txt",
                                                  "direct": "vmm_full_size_direct.txt",
                                                  "unrolled": "vmm_full_size_unrolled.txt",
                                                  "mlp_up": "vmm_full_size_mlp_up.txt",
                                                  "mlp_down": "vmm_full_size_mlp_down.txt"}[form])
    with open(out, "w") as f:
        f.write("# Oracle output of the full-size packed product (Algorithm 1 of App. C at the "
                + (f"MLP shape {plan.d_in} -> {plan.d_out},\n# level {level}" if mlp else "Table 2 shape\n# (S, d) = (32768, 4096)")
                + ") on integer plaintexts; written by make_vmm_full_size_golden.py"
                + (f" {form}\n# (sums of the baby steps kept in the extended basis"
                   + (", giant steps unrolled" if direct or unrolled else "")
                   + (", rotate-and-add ladders unrolled" if unrolled else "") + ").\n" if raised else ".\n"))
        f.write(f"shape: {' '.join(map(str, can.shape))}\n")
        f.write(f"level: {y.level}\n")
        f.write(f"rotations: {ctx.rot_count}\n")
        f.write(f"pt_mults: {ctx.ptmul_count}\n")
        f.write(f"sha256: {hashlib.sha256(can.tobytes()).hexdigest()}\n")
        for c in range(can.shape[0]):
            for l in range(can.shape[1]):
                f.write(f"head_{c}_{l}: {' '.join(str(int(v)) for v in can[c, l, :4])}\n")
    print("wrote", out, time.time() - t0)


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "plain")
