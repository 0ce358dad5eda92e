"""Dense brute force of the MoE layer in numpy fp64 -- test infrastructure only.

Written independently of moe_oracle.c to pin it on tiny inputs: every token is
pushed through EVERY expert, and a dense [T,E] gate matrix (zero outside the
top-k) weights the results.  The top-k here comes from sorting (-logit, index)
pairs, not from the oracle's running insertion.
"""
from __future__ import annotations

import numpy as np


def dense_gates(logits: np.ndarray, k: int) -> np.ndarray:
    """[T,E] fp64: softmax over all experts, zeroed outside the k winners,
    renormalised to sum 1."""
    lg = np.asarray(logits, dtype=np.float32).astype(np.float64)
    T, E = lg.shape
    g = np.zeros((T, E))
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-lg[t, e], e))
        win = order[:k]
        p = np.exp(lg[t] - lg[t].max())
        p /= p.sum()
        g[t, win] = p[win] / p[win].sum()
    return g


def dense_ffn(x: np.ndarray, w1: np.ndarray, w3: np.ndarray, w2: np.ndarray) -> np.ndarray:
    """One expert on all rows: (silu(x w1) * (x w3)) w2, fp64 numpy matmul."""
    a = x @ w1
    b = x @ w3
    return ((a / (1.0 + np.exp(-a))) * b) @ w2


def layer(x: np.ndarray, logits: np.ndarray, w1, w3, w2, k: int) -> np.ndarray:
    """x fp64 [T,d]; w1,w3 fp64 [E,d,f]; w2 fp64 [E,f,d] -> y fp64 [T,d]."""
    g = dense_gates(logits, k)
    y = np.zeros_like(x, dtype=np.float64)
    for e in range(w1.shape[0]):
        y += g[:, e:e + 1] * dense_ffn(x, w1[e], w3[e], w2[e])
    return y
