"""Seeded synthetic inputs with the shapes and value distributions of the benchmark configurations.

This module holds no arithmetic of the method itself (no transform, no coding, no packing): it
only draws random weight and activation tensors.  Both the HIP path and the CPU oracle are fed from the bytes produced
here, so that bit-exact comparisons never depend on two random generators agreeing.

Stand-in for real LLM checkpoints (none are available offline): weights are heavy-tailed
(Student-t, 4 degrees of freedom, times 0.02) with a few input channels blown up 20x, the pattern
of "outlier channels" the paper's introduction describes; activations are N(0,1) rounded to fp16
with 0.5 % of the channels scaled 10x.
"""
import numpy as np

MASTER_SEED = 20260327

# name -> list of (tensor name, N, K); M values live with the benchmark/test that uses them.
SHAPES = {
    "single": [("w", 2048, 2048)],
    "llama7b": [("attn", 4096, 4096), ("ffn_up", 11008, 4096), ("ffn_down", 4096, 11008)],
    "llama70b": [("attn_q", 8192, 8192), ("ffn_up", 28672, 8192), ("ffn_down", 8192, 28672), ("attn_kv", 1024, 8192)],
    "prefill": [("ffn_up", 14336, 4096), ("ffn_down", 4096, 14336)],
}

# One transformer layer of the 70B-shaped stream: (tensor name, N, K, copies per layer).
LLAMA70B_LAYER = [
    ("q", 8192, 8192, 1),
    ("kv", 1024, 8192, 2),
    ("o", 8192, 8192, 1),
    ("gate_up", 28672, 8192, 2),
    ("down", 8192, 28672, 1),
]
# One transformer layer of the 7B-shaped stream.
LLAMA7B_LAYER = [
    ("qkvo", 4096, 4096, 4),
    ("gate_up", 11008, 4096, 2),
    ("down", 4096, 11008, 1),
]


# The same layers as decode stages: the tensors of one stage read the same activations and are
# independent of each other (one grouped call); a stage needs the output of the stage before it.
LLAMA7B_STAGES = [
    [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096)],
    [("o", 4096, 4096)],
    [("gate", 11008, 4096), ("up", 11008, 4096)],
    [("down", 4096, 11008)],
]
LLAMA70B_STAGES = [
    [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192)],
    [("o", 8192, 8192)],
    [("gate", 28672, 8192), ("up", 28672, 8192)],
    [("down", 8192, 28672)],
]


def _rng(*key):
    words = [MASTER_SEED]
    for k in key:
        if isinstance(k, str):
            words.extend(k.encode())
        else:
            words.append(int(k))
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(words)))


def weights(N, K, *key, n_outlier_cols=None):
    """fp32 [N, K]: 0.02 * Student-t(nu=4); ``n_outlier_cols`` random input channels times 20
    (default round(0.001 K))."""
    g = _rng("W", N, K, *key)
    W = (0.02 * g.standard_t(4.0, size=(N, K))).astype(np.float32)
    if n_outlier_cols is None:
        n_outlier_cols = int(round(0.001 * K))
    if n_outlier_cols > 0:
        cols = g.choice(K, size=n_outlier_cols, replace=False)
        W[:, cols] *= np.float32(20.0)
    return W


def activations(M, K, *key, outlier_frac=0.005):
    """fp16 [M, K]: N(0,1), ``round(outlier_frac K)`` random channels times 10, rounded to fp16."""
    g = _rng("X", M, K, *key)
    X = g.standard_normal(size=(M, K)).astype(np.float32)
    n_out = int(round(outlier_frac * K))
    if n_out > 0:
        cols = g.choice(K, size=n_out, replace=False)
        X[:, cols] *= np.float32(10.0)
    return X.astype(np.float16)
