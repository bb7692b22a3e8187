"""Seeded synthetic inputs shaped like LLaMA linear layers.

Only random draws and reshaping live here: no rotation, selection, quantisation
or matmul of the method.  Tests and the bench feed the same arrays to the HIP
library and to the CPU checker.

Recipe (stands in for the LLaMA2-7B activations / weights the paper measured on):
  sigma_c = exp(N(0,1)) per input channel, shared by x and the calibration set
  x      = N(0,1) * sigma            -> fp16, [M, D]
  X_cal  = N(0,1) * sigma            fp64,    [N_cal, D]
  W      = N(0, 0.02^2), a uniformly random 0.1 % of entries multiplied by 10 -> fp16, [N, D]
Draw order is fixed: sigma, X_cal, x, W, outlier mask.
"""
from __future__ import annotations

import numpy as np


def make_layer(seed: int, M: int, D: int, N: int, n_cal: int):
    """Returns dict(sigma, X_cal fp64, x fp16, W fp16)."""
    rng = np.random.default_rng(seed)
    sigma = np.exp(rng.standard_normal(D))
    X_cal = rng.standard_normal((n_cal, D)) * sigma
    x = (rng.standard_normal((M, D)) * sigma).astype(np.float16)
    W = rng.standard_normal((N, D)) * 0.02
    mask = rng.random((N, D)) < 1e-3
    W = np.where(mask, W * 10.0, W).astype(np.float16)
    return dict(sigma=sigma, X_cal=X_cal, x=x, W=W)


def make_weight(seed: int, N: int, D: int) -> np.ndarray:
    """One more weight matrix with the W recipe above (for multi-layer benches)."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((N, D), dtype=np.float32) * np.float32(0.02)
    mask = rng.random((N, D), dtype=np.float32) < 1e-3
    return np.where(mask, W * np.float32(10.0), W).astype(np.float16)


def make_activations(seed: int, M: int, D: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    sigma = np.exp(rng.standard_normal(D))
    return (rng.standard_normal((M, D)) * sigma).astype(np.float16)


def random_orthogonal_blocks(seed: int, H: int, hd: int = 128) -> np.ndarray:
    """H random orthogonal hd x hd blocks (QR of Gaussian blocks), fp32.  Stands
    in for a PCA rotation where only the data layout and speed matter."""
    rng = np.random.default_rng(seed)
    out = np.empty((H, hd, hd), np.float32)
    for h in range(H):
        q, r = np.linalg.qr(rng.standard_normal((hd, hd)))
        out[h] = (q * np.sign(np.diag(r))).astype(np.float32)
    return out


def random_orthogonal_dense(seed: int, D: int, hd: int = 128) -> np.ndarray:
    """A dense D x D orthogonal matrix, fp32, built cheaply as B1 * P * B2 with
    B1, B2 block diagonal (random orthogonal hd x hd blocks) and P a stride
    permutation, so every entry is generally non-zero when hd*hd >= D."""
    assert D % hd == 0
    H = D // hd
    b1 = random_orthogonal_blocks(seed, H, hd).astype(np.float64)
    b2 = random_orthogonal_blocks(seed + 1, H, hd).astype(np.float64)
    # stride permutation: position i*H + h  <-  h*hd + i
    src = np.arange(D).reshape(H, hd).T.reshape(-1)
    Q = np.zeros((D, D), np.float32)
    # rows of B1 (block h1), permuted columns, then right-multiplied by B2 block by block
    for h1 in range(H):
        rows = np.zeros((hd, D))
        rows[:, h1 * hd:(h1 + 1) * hd] = b1[h1]
        rows = rows[:, src]
        for h2 in range(H):
            sl = slice(h2 * hd, (h2 + 1) * hd)
            Q[h1 * hd:(h1 + 1) * hd, sl] = (rows[:, sl] @ b2[h2]).astype(np.float32)
    return Q


def descending_spectrum(seed: int, D: int, blocks: int = 1) -> np.ndarray:
    """Positive 'eigenvalues', descending inside each of `blocks` equal runs
    (log-normal draws, sorted): a stand-in selection key for synthetic rotations."""
    rng = np.random.default_rng(seed)
    lam = np.exp(2.0 * rng.standard_normal(D)).reshape(blocks, D // blocks)
    return (-np.sort(-lam, axis=1)).reshape(-1)
