"""Seeded synthetic inputs for the Q-GaLore optimizer step.

This module only draws random tensors with the shapes, dtypes and structure of
the paper's workloads (LLaMA linear weights, low-rank-plus-noise bf16
gradients, orthonormal projection matrices).  It contains none of the method's
arithmetic: no quantizer, no hash generator, no optimizer maths.  It is the
one module that both the test oracle and the HIP path's callers share.
"""
from __future__ import annotations

import numpy as np

# tensor ids for the seed tuple
T_W, T_A, T_B, T_E, T_P, T_PNEW = range(6)

# (hidden, ffn, layers, rank) of the LLaMA-shaped workloads, by config index
LLAMA_SHAPES = {
    1: (768, 2048, 12, 256),     # 130M
    2: (1024, 2736, 24, 256),    # 350M
    3: (2048, 5461, 24, 512),    # 1B
    4: (4096, 11008, 32, 1024),  # 7B
}
MATRIX_KINDS = ("q", "k", "v", "o", "gate", "up", "down")

ADAM_BETA1, ADAM_BETA2, ADAM_EPS, LR, ALPHA = 0.9, 0.999, 1e-8, 1e-3, 0.25


def rng(config_seed: int, layer: int, kind: int, step: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([config_seed, layer, kind, step, tensor_id])))


def layer_shapes(config: int):
    """[(kind, m, n)] of the seven linear weights of one decoder layer."""
    h, f, _, _ = LLAMA_SHAPES[config]
    return [("q", h, h), ("k", h, h), ("v", h, h), ("o", h, h), ("gate", f, h), ("up", f, h), ("down", h, f)]


def config_matrices(config: int):
    """[(layer, kind_index, m, n, r)] of every linear weight of a config."""
    if config == 0:
        return [(0, 0, 512, 512, 128)]
    _, _, layers, r = LLAMA_SHAPES[config]
    return [(l, ki, m, n, r) for l in range(layers) for ki, (_, m, n) in enumerate(layer_shapes(config))]


def weight_f32(m: int, n: int, seed=0, layer=0, kind=0) -> np.ndarray:
    """W ~ N(0, std 0.02), fp32."""
    return (rng(seed, layer, kind, 0, T_W).standard_normal((m, n), dtype=np.float32) * np.float32(0.02))


def _to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (storage format of the gradient buffer),
    through torch's CPU cast."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def gradient_bf16(m: int, n: int, step: int, seed=0, layer=0, kind=0) -> np.ndarray:
    """G = A B^T + E stored as bf16 bit patterns (uint16 [m][n]); A is m x 16 and
    B is n x 16 with entries N(0, std 0.01), E has entries N(0, std 1e-4); redrawn
    for every step."""
    A = rng(seed, layer, kind, step, T_A).standard_normal((m, 16), dtype=np.float32) * np.float32(0.01)
    B = rng(seed, layer, kind, step, T_B).standard_normal((n, 16), dtype=np.float32) * np.float32(0.01)
    E = rng(seed, layer, kind, step, T_E).standard_normal((m, n), dtype=np.float32) * np.float32(1e-4)
    return _to_bf16_bits(A @ B.T + E)


def projection_f32(m: int, r: int, seed=0, layer=0, kind=0, tensor_id=T_P) -> np.ndarray:
    """P = Q-factor (numpy.linalg.qr, fp64) of a seeded Gaussian m x r, as fp32."""
    g = rng(seed, layer, kind, 0, tensor_id).standard_normal((m, r))
    q, _ = np.linalg.qr(g)
    return np.ascontiguousarray(q.astype(np.float32))


def perturbed_projection_f32(P: np.ndarray, eps: float, seed=0, layer=0, kind=0) -> np.ndarray:
    """Q-factor of P + eps * Gaussian: a neighbouring subspace, for sweeping the
    cosine similarity across the refresh threshold."""
    g = rng(seed, layer, kind, 0, T_PNEW).standard_normal(P.shape)
    q, rr = np.linalg.qr(P.astype(np.float64) + eps * g)
    q = q * np.sign(np.diag(rr))[None, :]           # keep column orientation
    return np.ascontiguousarray(q.astype(np.float32))
