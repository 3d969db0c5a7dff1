"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Only random tensors of the workloads' shapes live here -- none of the method's arithmetic.
The float tensors stand in for Llama-3-8B activations, weights and cached keys/values: the
cost of modular arithmetic does not depend on the values, so Gaussian / uniform tensors of
the right shape exercise the same path as trained weights would.
"""
import numpy as np


def vmm_inputs(seed, d_in, d_out, x_dist="normal", w_sigma=0.02):
    """Activation row x[d_in] and weight matrix W[d_in, d_out]."""
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, d_in) if x_dist == "uniform" else rng.normal(0, 1, d_in)
    W = rng.normal(0, w_sigma, (d_in, d_out))
    return x, W


def attention_inputs(seed, heads, kv_heads, dim, ntok):
    """Query q[heads, dim], cached K and V [ntok, heads, dim] (kv_heads distinct heads, each
    shared by heads/kv_heads query heads), scores s[heads, ntok] with rows summing to 1."""
    rng = np.random.default_rng(seed)
    q = rng.normal(0, 1, (heads, dim))
    rep = heads // kv_heads
    K = np.repeat(rng.normal(0, 1, (ntok, kv_heads, dim)), rep, axis=1)
    V = np.repeat(rng.normal(0, 1, (ntok, kv_heads, dim)), rep, axis=1)
    s = rng.uniform(0, 1, (heads, ntok))
    s /= s.sum(axis=1, keepdims=True)
    return q, K, V, s
