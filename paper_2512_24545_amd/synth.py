"""Seeded synthetic MDBF layers and activations.

This module only draws random inputs (numpy, host side).  It contains none of
the method's arithmetic and is the single piece of code that both the HIP path's
callers and the CPU oracle's callers may share: the same arrays are handed to
both sides.

A layer is a dict with
    m, n, k, l             shapes (What is m x n, inner rank k, envelope rank l)
    SA (m,k) int8, SB (k,n) int8          sign bases, entries +-1
    A (m,l), Q (k,l), G (k,l), B (n,l)    envelope factors, float32 arrays whose
                                           values are exactly representable in
                                           `env_dtype`
    env_dtype                              "f16" | "bf16" | "f32"
Activations are float32 arrays whose values are exact in `x_dtype`.

The shapes and distributions follow the benchmark configurations: i.i.d. +-1
signs with p = 1/2, half-normal envelopes (|N(0,1)|*0.02 + 1e-3 for the LLaMA-7B
shaped layers, |N(0,1)| + 0.1 for the toy and prefill cases), N(0,1) activations.
They stand in for quantized LLaMA-7B projections: throughput of the forward
product does not depend on the values.
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f16", "bf16", "f32")


def round_to_dtype(a, dtype):
    """Round a float array to the nearest value of `dtype`, returned as float32."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "f32":
        return a.copy()
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = a.view(np.uint32).astype(np.uint64)
        # round to nearest even on the upper 16 bits
        u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
        return (u.astype(np.uint32) << 16).view(np.float32).reshape(a.shape)
    raise ValueError(f"unknown dtype {dtype}")


def random_signs(rng, rows, cols):
    return (rng.integers(0, 2, size=(rows, cols), dtype=np.int8) * 2 - 1).astype(np.int8)


def make_layer(m, n, k, l, seed, env_dtype="f16", env_kind="llama", signed_env=False):
    """env_kind "llama": |N(0,1)|*0.02 + 1e-3;  "unit": |N(0,1)| + 0.1;  "ones": all 1.
    signed_env flips the sign of each envelope entry with probability 1/2."""
    rng = np.random.default_rng(seed)
    SA = random_signs(rng, m, k)
    SB = random_signs(rng, k, n)

    def env(rows):
        g = np.abs(rng.standard_normal((rows, l)))
        if env_kind == "llama":
            e = g * 0.02 + 1e-3
        elif env_kind == "unit":
            e = g + 0.1
        elif env_kind == "ones":
            e = np.ones((rows, l))
        else:
            raise ValueError(env_kind)
        if signed_env:
            e = e * (rng.integers(0, 2, size=(rows, l)) * 2 - 1)
        return round_to_dtype(e, env_dtype)

    A = env(m)
    Q = env(k)
    G = env(k)
    B = env(n)
    return dict(m=m, n=n, k=k, l=l, SA=SA, SB=SB, A=A, Q=Q, G=G, B=B, env_dtype=env_dtype)


def structured_weight(rows, cols, seed, decay=0.7, scale=0.02):
    """A dense weight matrix with a decaying spectrum (singular values ~ i^-decay), the input of a
    quantisation run: Gaussian factors around a power-law diagonal, scaled to weight-like magnitudes."""
    rng = np.random.default_rng(seed)
    r = min(rows, cols)
    core = rng.standard_normal((rows, r)) @ np.diag(1.0 / np.arange(1, r + 1) ** decay) @ rng.standard_normal((r, cols))
    return scale * core / np.sqrt(r)


def make_activations(n, T, seed, x_dtype="f16", kind="normal"):
    """kind "normal": N(0,1);  "ternary": i.i.d. from {-1,0,+1} (exact-integer tests)."""
    rng = np.random.default_rng(seed)
    if kind == "normal":
        x = rng.standard_normal((T, n))
    elif kind == "ternary":
        x = rng.integers(-1, 2, size=(T, n)).astype(np.float64)
    else:
        raise ValueError(kind)
    return round_to_dtype(x, x_dtype)


def normal_block(rows, cols, seed):
    """Seeded N(0,1) block (fp32): the start block of the subspace iteration inside mdbf_msvid, which draws no
    random numbers itself."""
    return np.random.default_rng(seed).standard_normal((rows, cols)).astype(np.float32)


# ---------------------------------------------------------------------------
# the benchmark configurations
# ---------------------------------------------------------------------------
def config_toy():
    """256x256, k=128, l=4, fp32 envelopes |N|+0.1, one fp32 token, seed 0."""
    layer = make_layer(256, 256, 128, 4, seed=0, env_dtype="f32", env_kind="unit")
    X = make_activations(256, 1, seed=1000, x_dtype="f32")
    return layer, X


def config_attn_decode(seed=2, T=1):
    """LLaMA-7B attention projection: 4096x4096, k=2656, l=16 (about 1.5 bits/weight)."""
    layer = make_layer(4096, 4096, 2656, 16, seed=seed, env_dtype="f16", env_kind="llama")
    X = make_activations(4096, T, seed=seed + 1000, x_dtype="f16")
    return layer, X


MLP_SHAPES = {
    "gate": (11008, 4096, 4096, 30),
    "up": (11008, 4096, 4096, 31),
    "down": (4096, 11008, 4096, 32),
}


def config_mlp_decode(which, T=1):
    """LLaMA-7B MLP projections in decode: gate/up 11008x4096, down 4096x11008, k=4096, l=16."""
    m, n, k, seed = MLP_SHAPES[which]
    layer = make_layer(m, n, k, 16, seed=seed, env_dtype="f16", env_kind="llama")
    X = make_activations(n, T, seed=seed + 1000, x_dtype="f16")
    return layer, X


def config_prefill(T=2048, x_dtype="f16", env_kind="unit"):
    """Prefill on the 4096x4096, k=2656, l=16 layer; envelopes drawn as in the toy config."""
    layer = make_layer(4096, 4096, 2656, 16, seed=4, env_dtype="f16", env_kind=env_kind)
    X = make_activations(4096, T, seed=1004, x_dtype=x_dtype)
    return layer, X


# inner ranks of the 32-layer stack per budget: (l, k for 4096x4096, k for 11008<->4096)
STACK_BUDGETS = {
    "1.0": (8, 1856, 2816),
    "1.5": (16, 2656, 4096),
    "2.0": (16, 3616, 5536),
}
STACK_MATS = ("q", "k", "v", "o", "gate", "up", "down")


def stack_matrix_spec(budget, layer_idx, mat_idx):
    """Shape and seed of one of the 224 matrices of the synthetic decoder stack."""
    l, k_attn, k_mlp = STACK_BUDGETS[budget]
    name = STACK_MATS[mat_idx]
    if name in ("q", "k", "v", "o"):
        m, n, k = 4096, 4096, k_attn
    elif name in ("gate", "up"):
        m, n, k = 11008, 4096, k_mlp
    else:
        m, n, k = 4096, 11008, k_mlp
    bidx = list(STACK_BUDGETS).index(budget)
    seed = 5000 + 100 * bidx + 7 * layer_idx + mat_idx
    return dict(m=m, n=n, k=k, l=l, seed=seed, name=name)


def stack_matrix(budget, layer_idx, mat_idx, T=1):
    sp = stack_matrix_spec(budget, layer_idx, mat_idx)
    layer = make_layer(sp["m"], sp["n"], sp["k"], sp["l"], seed=sp["seed"])
    X = make_activations(sp["n"], T, seed=sp["seed"] + 100000)
    return layer, X
