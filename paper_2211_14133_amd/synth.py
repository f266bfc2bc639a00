"""Seeded synthetic inputs with the shapes of BERT K-FAC work (no method arithmetic here).

The paper's workload is BERT pre-training (micro-batches of 32 sequences of
128 tokens; d_model/d_ff = 768/3072 for BERT-Base and 1024/4096 for
BERT-Large, Table 3 of the appendix).  Its data set is not available, so the
tensors below stand in for it: layer inputs are N(0,1) draws, except the input
of the second feed-forward linear which is GELU(N(0,1)); output errors are
N(0, 1e-6) draws.  Every element is a pure function of (seed, tensor id,
element index), so any consumer sees the same bits.

This module only produces inputs.  The curvature, inversion and precondition
arithmetic lives in the HIP library and, separately, in the test oracle.
"""
import numpy as np
from scipy.special import erf

SEED = 221114133
DAMPING = 1e-3

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x):
    """One splitmix64 output per uint64 counter value (vectorised)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def standard_normal(tensor_id, count, seed=SEED):
    """``count`` float64 N(0,1) values: Box-Muller on two counter-based uniforms."""
    i = np.arange(count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        base = np.uint64(tensor_id) * np.uint64(1 << 40) + np.uint64(2) * i
        h0 = _splitmix64(np.uint64(seed) ^ base)
        h1 = _splitmix64(np.uint64(seed) ^ (base + np.uint64(1)))
    u1 = ((h0 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
    u2 = (h1 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def gelu_exact(x):
    """x * Phi(x) with the error function, float64."""
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def round_to_bf16(x32):
    """Round float32 values to the nearest bfloat16 (ties to even), kept as float32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32).reshape(np.shape(x32))


def tensor_id(cfg, block, layer, microbatch, is_error):
    return cfg * 10 ** 6 + block * 10 ** 4 + layer * 10 ** 2 + microbatch * 2 + (1 if is_error else 0)


def activations(cfg, block, layer, microbatch, tokens, d, gelu=False, bf16=False, seed=SEED):
    """Layer input ``[tokens, d]`` float32 (bf16-representable if ``bf16``)."""
    z = standard_normal(tensor_id(cfg, block, layer, microbatch, False), tokens * d, seed)
    if gelu:
        z = gelu_exact(z)
    x = z.astype(np.float32).reshape(tokens, d)
    return round_to_bf16(x) if bf16 else x


def errors(cfg, block, layer, microbatch, tokens, d, scale=1e-3, bf16=False, seed=SEED):
    """Output errors ``[tokens, d]`` float32, N(0, scale^2)."""
    z = standard_normal(tensor_id(cfg, block, layer, microbatch, True), tokens * d, seed) * scale
    e = z.astype(np.float32).reshape(tokens, d)
    return round_to_bf16(e) if bf16 else e


def weight_gradient(es, xs):
    """The gradient handed to precondition: mean over all tokens of e x^T, rounded once to float32.

    This is an input of the K-FAC work (the backward pass produces it), not part of it.
    """
    n = sum(x.shape[0] for x in xs)
    g = np.zeros((es[0].shape[1], xs[0].shape[1]))
    for e, x in zip(es, xs):
        g += e.astype(np.float64).T @ x.astype(np.float64)
    return (g / n).astype(np.float32)


def block_layers(d_model, d_ff):
    """(name, d_in, d_out, gelu_input) of the six linears of a transformer encoder block."""
    return [
        ("q", d_model, d_model, False),
        ("k", d_model, d_model, False),
        ("v", d_model, d_model, False),
        ("o", d_model, d_model, False),
        ("ffn1", d_model, d_ff, False),
        ("ffn2", d_ff, d_model, True),
    ]


#: The workloads named by the benchmark definition.
CONFIGS = {
    1: dict(name="single-64", layers=[("fc", 64, 64, False)], blocks=1, tokens=256, n_micro=1, bf16=False),
    2: dict(name="bert-base-block", layers=block_layers(768, 3072), blocks=1, tokens=4096, n_micro=1, bf16=False),
    3: dict(name="bert-large-block", layers=block_layers(1024, 4096), blocks=1, tokens=4096, n_micro=1, bf16=False),
    4: dict(name="bert-large-stage", layers=block_layers(1024, 4096), blocks=6, tokens=4096, n_micro=8, bf16=False),
    5: dict(name="stress-2048-8192", layers=block_layers(2048, 8192), blocks=1, tokens=8192, n_micro=1, bf16=True),
    # the longer sequences of the paper's table of performance-model figures (appendix): same layer
    # shapes as BERT-Large, 32 sequences of 512 (T5-Large) and of 2048 (OPT-350M) tokens per micro-batch
    6: dict(name="t5-large-block-s512", layers=block_layers(1024, 4096), blocks=1, tokens=16384, n_micro=1, bf16=False),
    7: dict(name="opt-350m-block-s2048", layers=block_layers(1024, 4096), blocks=1, tokens=65536, n_micro=1, bf16=False),
}


def hadamard_columns(n, d):
    """First ``d`` columns of the n x n Sylvester-Hadamard matrix (+-1), n a power of two."""
    assert n & (n - 1) == 0 and d <= n
    r = np.arange(n, dtype=np.int64)[:, None]
    c = np.arange(d, dtype=np.int64)[None, :]
    bits = r & c
    par = np.zeros_like(bits)
    while bits.any():
        par ^= bits & 1
        bits >>= 1
    return (1.0 - 2.0 * par).astype(np.float32)
