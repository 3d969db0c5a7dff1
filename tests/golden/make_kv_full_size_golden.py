"""Writes tests/golden/kv_full_size.txt by running ONLY the oracle.

Full-size parity case of the products against the encrypted KV cache (Sec. 5.1-5.3) and of the cache
appends (Sec. 5.1 "K Cache Update", Sec. 5.2 "V Cache Update", Sec. 5.4 for a token group): ring n = 2^16
with 24 x 50-bit + 4 x 60-bit primes (benchmark configuration 2), Llama-3-8B attention shapes (H = 32
heads of E = 128 dims, t = 8 tokens per K ciphertext, 128 V ciphertexts with 16 baby x 8 giant steps),
cache one level below the top, as `bench.py --workload attention` runs it.

Scenario (every ciphertext and every rotation has its full size):
  1. one token group (tokens 0..7) and two single tokens (8, 9: residues 0 and 1) are appended to an
     empty cache; K ciphertexts 0, 1 and all 128 V ciphertexts are recorded;
  2. q K^T in the printed order (per K ciphertext: product, relinearisation, rescale, seven rotate-and-add
     steps, mask) over the two K ciphertexts;
  3. scores V over the 128 V ciphertexts, in the printed order and with giant steps and residue ladder
     unrolled in the extended basis;
  4. K ciphertexts 2..15 are loaded and q K^T runs over 16 K ciphertexts with the copy mask in front of all
     128 terms of the sum over the dims (the form the attention workload of bench.py times; 16 x 128 masked
     products are enough for the library to take the transform along the copy index, as it does there).

Plaintexts, masks, queries, scores and cached vectors enter as integer coefficient polynomials drawn from a
seeded integer generator: ciphertext-level parity does not care what they encode, and integers cross
between machines bit for bit, which encoded floats need not.

The fixture stores, per recorded ciphertext, a SHA-256 of its canonical form and the first coefficients of
its first and last limb.  Run from the repository root (about a quarter of an hour on 8 cores, ~35 GiB):
    python tests/golden/make_kv_full_size_golden.py
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

H, E, R_I = 32, 128, 16
SEED_SK, SEED_EVK = 1, 2
GROUP_SEEDS = (100, 500)              # token group 0: key / value polynomial seeds (encryption seed = 1000 + that)
TOKENS = (8, 9)                       # single appends: polynomial seeds 100 + n / 500 + n
LOADED_K = tuple(range(2, 16))        # K ciphertexts loaded for the 16-ciphertext product: seed 200 + c
SEED_Q, SEED_S = 10, 50
MASK_SEEDS = {0: 900, 1: 901, 2: 902, 3: 903, 4: 904}
SHARED = 128
OUT = os.path.join(ROOT, "tests", "golden", "kv_full_size.txt")


def poly(n, seed, bits=48):
    """Integer polynomial with uniform coefficients below 2^bits in magnitude."""
    return np.random.default_rng(seed).integers(-2 ** bits, 2 ** bits, n, dtype=np.int64)


def all_steps(S):
    """Every rotation amount the scenario uses (t = 8, B = H t = 256 slots per copy)."""
    t = S // (H * E)
    B = H * t
    steps = [-(1 << i) for i in range(3)] + [k * B for k in range(1, E)] + list(range(1, t))
    return steps + [-(g * R_I * B) for g in range(1, E // R_I)]


def digest(can):
    return hashlib.sha256(np.ascontiguousarray(can).tobytes()).hexdigest()


def record_lines(name, can):
    rows = [f"{name}_shape: {' '.join(map(str, can.shape))}", f"{name}_sha256: {digest(can)}"]
    for c in range(can.shape[0]):
        for l in (0, can.shape[1] - 1):
            rows.append(f"{name}_head_{c}_{l}: {' '.join(str(int(v)) for v in can[c, l, :4])}")
    return rows


def run_oracle(log=print):
    from oracle import ckks, packing, params, vmm
    from oracle.ckks import Pt
    t0 = time.time()
    prm = params.config2()
    ctx = ckks.Context(prm)
    n, L = ctx.n, prm.L
    lv = L - 1
    lay = packing.KvLayout(ctx.S, H, E, R_I)
    sk = ctx.keygen_secret(SEED_SK)
    keys = ctx.keygen_rotations(sk, all_steps(ctx.S), SEED_EVK, with_relin=True)
    log("keys", len(keys), round(time.time() - t0))
    ops = vmm.CkksOps(ctx, keys)
    bases = {0: poly(n, MASK_SEEDS[0]), **{k: poly(n, MASK_SEEDS[k]) for k in (1, 2, 3, 4)}}

    def mask(kind, shift_right, level):
        idx = ctx.q_idx(level)
        coeff = ctx.automorphism_coeff(ctx.from_i64(bases[kind], idx), idx, ctx.galois(-shift_right))
        return Pt(ctx.ntt(coeff, idx), level, float(ctx.mod[level]))

    def enc(seed, level):
        ct = ctx.encrypt(sk, ctx.pt_from_coeffs(poly(n, seed), L, prm.scale), 1000 + seed)
        return ctx.level_drop(ct, level)

    out = {}
    okc, ovc = [], [None] * E
    # 1. appends
    vmasks = [mask(4, lay.slot((0 - k) % E, 0, 0) + lay.v_shift(k), lv + 1) for k in range(E)]
    vmm.kv_append_group(ops, lay, okc, ovc, 0, enc(GROUP_SEEDS[0], L), enc(GROUP_SEEDS[1], L), mask(3, 0, lv + 1), vmasks)
    log("group append", round(time.time() - t0))
    for tok in TOKENS:
        c, tau = tok // lay.t, tok % lay.t
        vmasks = [mask(2, lay.slot((c - k) % E, 0, tau) + lay.v_shift(k), lv + 1) for k in range(E)]
        vmm.kv_append(ops, lay, okc, ovc, tok, enc(100 + tok, L), enc(500 + tok, L), mask(1, tau, lv + 1), vmasks)
        log("append", tok, round(time.time() - t0))
    for c in range(2):
        out[f"K{c}"] = ctx.canonical(okc[c])
    hv = hashlib.sha256()
    for k in range(E):
        can = ctx.canonical(ovc[k])
        hv.update(can.tobytes())
        if k in (0, 17, E - 1):
            out[f"V{k}"] = can
    out["V_all_sha256"] = hv.hexdigest()
    # 2. q K^T as printed, two K ciphertexts
    cq = enc(SEED_Q, lv)
    qmask = [mask(0, b * H * lay.t, lv - 1) for b in range(E)]
    out["qk_printed"] = ctx.canonical(vmm.qk_scores(ops, lay, cq, okc, qmask[:2]))
    log("qk printed", round(time.time() - t0))
    # 3. scores V, printed and unrolled
    cs = enc(SEED_S, lv)
    out["sv_printed"] = ctx.canonical(vmm.score_times_v(ops, lay, cs, ovc))
    log("sv printed", round(time.time() - t0))
    out["sv_unrolled"] = ctx.canonical(vmm.score_times_v_unrolled(ctx, keys, lay, cs, ovc))
    log("sv unrolled", round(time.time() - t0))
    # 4. sixteen K ciphertexts, copy mask in front of the whole sum over the dims
    for c in LOADED_K:
        okc.append(enc(200 + c, lv))
    out["qk_shared"] = ctx.canonical(vmm.qk_scores_shared(ctx, keys, lay, cq, okc, qmask, SHARED))
    log("qk shared", round(time.time() - t0))
    return out


def main():
    out = run_oracle(lambda *a: print(*a, flush=True))
    with open(OUT, "w") as f:
        f.write("# Oracle outputs of the full-size cache scenario (appends of Sec. 5.1 / 5.2 / 5.4, q K^T of Sec. 5.1 / 5.3 in\n"
                "# the printed order and with the copy mask first, scores V of Sec. 5.2 / 5.3 in the printed order and\n"
                "# unrolled) on integer plaintexts; written by make_kv_full_size_golden.py.\n")
        for name, val in out.items():
            if isinstance(val, str):
                f.write(f"{name}: {val}\n")
            else:
                f.write("\n".join(record_lines(name, val)) + "\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
