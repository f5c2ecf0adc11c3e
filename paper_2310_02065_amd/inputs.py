"""Seeded synthetic inputs shared by the tests, the CPU oracle legs and the benchmark.

This module only DRAWS inputs (weights, a V:N:M-legal mask, activations); it contains none of
the format's or the product's arithmetic, and imports neither the oracle nor the HIP binding.

Recipe (stands in for the pruned BERT / random-weight GPT-3 layers the paper measures on --
V:N:M gives every row the same number of kept entries, so only the shape and the randomness of
the selected columns matter): numpy Generator(PCG64), one child stream for the structure, one
for the values of A, one for B.
  structure: per V x M block choose 4 of the M columns uniformly without replacement, sorted;
             per row of the block keep 2 of those 4 uniformly.  M = 4 keeps all four columns.
  values:    A = fp16(sigma_a * N(0,1)) on the WHOLE R x K matrix (entries outside the mask are
             random too: compression has to ignore them); B = fp16(N(0,1)).
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20231002

# name -> (R, K, C, V, M, sigma_a); the transformer-shaped workloads of the benchmark
CONFIGS = {
    "tiny":        (256, 256, 64, 64, 8, 1.0),
    "bert_base":   (3072, 768, 4096, 64, 8, 0.02),
    "bert_large":  (4096, 1024, 16384, 128, 16, 0.02),
    "gpt3":        (49152, 12288, 2048, 128, 32, 0.02),
}
SWEEP_SHAPE = (8192, 8192)            # R, K of the sparsity sweep
SWEEP_C = (256, 2048, 8192)
SWEEP_V = (64, 128)
SWEEP_M = (4, 8, 16, 32, 64, 128)


def _streams(seed: int):
    s_struct, s_a, s_b = np.random.SeedSequence(seed).spawn(3)
    mk = lambda s: np.random.Generator(np.random.PCG64(s))
    return mk(s_struct), mk(s_a), mk(s_b)


def config_seed(config_index: int, trial: int = 0) -> int:
    return BASE_SEED + 1000 * config_index + trial


def gen_mask(R: int, K: int, V: int, M: int, rng: np.random.Generator) -> np.ndarray:
    """uint8 R x K mask with the V:N:M structure described in the module docstring."""
    assert R % V == 0 and K % M == 0 and M >= 4
    Rb, G = R // V, K // M
    cols = np.sort(np.argsort(rng.random((Rb, G, M), dtype=np.float32), axis=-1)[..., :4], axis=-1)
    pick = np.argsort(rng.random((Rb, V, G, 4), dtype=np.float32), axis=-1)[..., :2]
    chosen = np.take_along_axis(np.broadcast_to(cols[:, None], (Rb, V, G, 4)), pick, axis=-1)
    mask = np.zeros((Rb, V, G, M), dtype=np.uint8)
    np.put_along_axis(mask, chosen, np.uint8(1), axis=-1)
    return mask.reshape(R, K)


def gen_problem(R, K, C, V, M, sigma_a=1.0, seed=BASE_SEED):
    """Returns (A_bits uint16 RxK, mask uint8 RxK, B_bits uint16 KxC)."""
    r_struct, r_a, r_b = _streams(seed)
    mask = gen_mask(R, K, V, M, r_struct)
    A = (r_a.standard_normal((R, K), dtype=np.float32) * np.float32(sigma_a)).astype(np.float16)
    B = r_b.standard_normal((K, C), dtype=np.float32).astype(np.float16)
    return A.view(np.uint16), mask, B.view(np.uint16)


def gen_B(K, C, seed=BASE_SEED):
    _, _, r_b = _streams(seed)
    return r_b.standard_normal((K, C), dtype=np.float32).astype(np.float16).view(np.uint16)
