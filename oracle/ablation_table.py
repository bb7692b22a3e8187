"""Synthetic analogue of the paper's two ablations, computed by the CPU oracle alone.

TEST INFRASTRUCTURE ONLY (like everything under oracle/).  Prints two markdown tables:

  1. salient-channel ablation appendix: which K rotated channels stay fp16 -- Top (the method),
     Bottom, Random (K consecutive channels from a random start, mean over several starts) and
     Top & Bottom (the channels of both, 2 K in fp16) -- scored by the relative output error
     ||y_stored - x W^T||_F / ||x W^T||_F on held-out activations (the paper scores perplexity,
     which needs its model and dataset);
  2. head-wise ablation appendix: one PCA per head (Eq. 6) against one global PCA over the
     concatenated heads (Eq. 8) for an output-projection-shaped layer, same K and bits, with few
     (D / 2) and with many (2 D) calibration rows: a 128 x 128 second moment is estimated from
     four times as many rows per dimension as the 512 x 512 one, which is where the head-wise
     rotation gains on this data; with plenty of rows and independent heads the two coincide.

Inputs are the seeded log-normal-channel activations and Gaussian-with-outliers weights of
paper_2506_13472_amd/synth.py; nothing of the HIP library is used.

    python -m oracle.ablation_table [--seeds 0,1,2]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from oracle import rosaq_oracle as O                      # noqa: E402
from paper_2506_13472_amd import synth                    # noqa: E402


def selection_ablation(seed: int, D: int = 512, N: int = 128, K: int = 128, bits: int = 3,
                       n_cal: int = 1024, M: int = 256, starts: int = 8) -> dict:
    """Relative output error of each selection rule on one synthetic layer (layer-wise PCA)."""
    lay = synth.make_layer(seed, M, D, N, n_cal)
    Q, lam = O.pca_full(lay["X_cal"], "lapack" if D > 256 else "jacobi")
    Q32 = Q.astype(np.float32)

    def err(K_, rule, arg=0):
        p = O.pack(lay["W"], Q32, lam, K_, bits, O.MODE_FULL, rule=rule, arg=arg)
        return O.quality_report(lay["x"], lay["W"], Q32, p)

    rng = np.random.default_rng(1000 + seed)
    random_starts = rng.integers(0, D - K + 1, size=starts)
    return {
        "Top": err(K, O.RULE_TOP),
        "Bottom": err(K, O.RULE_BOTTOM),
        "Random": float(np.mean([err(K, O.RULE_CONSECUTIVE, int(a)) for a in random_starts])),
        "Top & Bottom": err(2 * K, O.RULE_TOP_AND_BOTTOM),
        "none (all low-bit)": err(0, O.RULE_TOP),
    }


def correlated_heads(seed: int, rows: int, H: int, hd: int, rank: int = 8) -> np.ndarray:
    """Activations of H heads: per head a few strong latent directions (what one attention head
    writes) on top of the log-normal per-channel noise of the usual recipe; heads independent."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, H * hd))
    for h in range(H):
        sigma = np.exp(rng.standard_normal(hd))
        basis = rng.standard_normal((rank, hd)) * np.exp(rng.standard_normal((rank, 1)) + 1.0)
        out[:, h * hd:(h + 1) * hd] = rng.standard_normal((rows, rank)) @ basis + \
            rng.standard_normal((rows, hd)) * sigma
    return out


def headwise_ablation(seed: int, H: int = 4, hd: int = 128, N: int = 128, K: int = 128,
                      bits: int = 3, n_cal: int = 512, M: int = 256) -> dict:
    """Head-wise PCA (Eq. 6) against one global PCA (Eq. 8) on an output-projection-shaped layer:
    the same calibration rows, the same K fp16 channels in total, the same bits."""
    D = H * hd
    gen = correlated_heads(seed, n_cal + M, H, hd)
    X_cal = gen[:n_cal]
    x = gen[n_cal:].astype(np.float16)
    W = synth.make_weight(500 + seed, N, D)
    Qb, lam_b = O.pca_headwise(X_cal, hd, "jacobi")
    Qb32 = Qb.astype(np.float32)
    Qg, lam_g = O.pca_full(X_cal, "lapack")
    Qg32 = Qg.astype(np.float32)
    p_head_global_topk = O.pack(W, Qb32, lam_b, K, bits, O.MODE_HEADWISE)
    p_head_per_head = O.pack(W, Qb32, lam_b, K, bits, O.MODE_HEADWISE, rule=O.RULE_TOP_PER_HEAD)
    p_global = O.pack(W, Qg32, lam_g, K, bits, O.MODE_FULL)
    p_none = O.pack(W, None, np.abs(X_cal).mean(axis=0), K, bits, O.MODE_NONE)
    return {
        "head-wise PCA, K/H per head": O.quality_report(x, W, Qb32, p_head_per_head),
        "head-wise PCA, top-K over all heads": O.quality_report(x, W, Qb32, p_head_global_topk),
        "global PCA": O.quality_report(x, W, Qg32, p_global),
        "no rotation (top-K by magnitude)": O.quality_report(x, W, None, p_none),
    }


def table(title: str, rows: list[dict], seeds) -> str:
    keys = list(rows[0].keys())
    head = "| " + title + " | " + " | ".join(f"seed {s}" for s in seeds) + " | mean |"
    sep = "|---|" + "---|" * (len(seeds) + 1)
    lines = [head, sep]
    for k in keys:
        vals = [r[k] for r in rows]
        lines.append("| " + k + " | " + " | ".join(f"{v:.4f}" for v in vals) + f" | {np.mean(vals):.4f} |")
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seeds", default="0,1,2")
    args = ap.parse_args()
    seeds = [int(s) for s in args.seeds.split(",")]
    print("relative output error ||y_stored - x W^T||_F / ||x W^T||_F, INT3 g128, K = 128 "
          "(Top & Bottom: 256), held-out activations\n")
    print(table("fp16 channels (layer-wise PCA, D = 512)", [selection_ablation(s) for s in seeds], seeds))
    print()
    for n_cal in (256, 1024):
        print(table(f"rotation (4 heads x 128, output projection, {n_cal} calibration rows)",
                    [headwise_ablation(s, n_cal=n_cal) for s in seeds], seeds))
        print()


if __name__ == "__main__":
    main()
