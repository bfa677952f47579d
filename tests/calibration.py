"""Harness-side stand-in for the cheap, closed-form part of the paper's calibration (Alg. 2,
App. A): structured synthetic K/V whose redundancy resembles what Sec. 3.1 describes (keys of
neighbouring vision tokens nearly parallel, values of low rank along the sequence axis), and
parameters fitted to it.  Not part of the library or of the oracle: numpy only.

  * U[h]     = top-m left singular vectors of the centred calibration values stacked along the
               channel axis (Sec. 3.1: PCA basis along the sequence dimension), mu[h] their mean row;
  * M        = m evenly spaced positions (the paper learns the mask; any fixed mask serves here);
  * theta[h] = least-squares map from the retained key rows to all key rows on the calibration
               blocks, theta[h]^T = K_cal pinv(K_cal[M]).
"""
from __future__ import annotations

import numpy as np


def structured_blocks(rng, n_blocks, n, d, rank, noise):
    """[n_blocks, n, d] blocks X = A G + noise with a smooth sequence-axis basis A [n, rank]
    shared by all blocks (returned as well) and block-specific mixing G [rank, d]."""
    walk = np.cumsum(rng.standard_normal((n, rank)), axis=0)          # neighbouring rows are close
    A = walk / np.linalg.norm(walk, axis=0, keepdims=True) * np.sqrt(n)
    G = rng.standard_normal((n_blocks, rank, d)) / np.sqrt(rank)
    X = A[None] @ G + noise * rng.standard_normal((n_blocks, n, d))
    return X, A


def make_structured_kv(seed, B, Hkv, n, I, d, rank, noise, Ak=None, Av=None, mu=None):
    """K, V [B, Hkv, I*n, d] (float64).  The sequence-axis bases are per KV head and shared by all
    blocks and batch elements; pass the ones returned by an earlier call to draw held-out data from
    the same distribution."""
    rng = np.random.default_rng(seed)
    K = np.empty((B, Hkv, I * n, d))
    V = np.empty((B, Hkv, I * n, d))
    new = Ak is None
    if new:
        Ak, Av = np.empty((Hkv, n, rank)), np.empty((Hkv, n, rank))
        mu = rng.standard_normal((Hkv, d)) * 0.5
    for h in range(Hkv):
        Xk, a = structured_blocks(rng, B * I, n, d, rank, noise)
        Xv, b = structured_blocks(rng, B * I, n, d, rank, noise)
        if new:
            Ak[h], Av[h] = a, b
        else:       # same bases, fresh mixing and noise
            Gk = rng.standard_normal((B * I, rank, d)) / np.sqrt(rank)
            Gv = rng.standard_normal((B * I, rank, d)) / np.sqrt(rank)
            Xk = Ak[h][None] @ Gk + noise * rng.standard_normal((B * I, n, d))
            Xv = Av[h][None] @ Gv + noise * rng.standard_normal((B * I, n, d))
        K[:, h] = Xk.reshape(B, I * n, d)
        V[:, h] = (Xv + mu[h]).reshape(B, I * n, d)
    return K, V, Ak, Av, mu


def fit_params(K, V, n, m):
    """Closed-form calibration on K, V [B, Hkv, I*n, d]: returns key_idx [m], theta [Hkv, m, n],
    U [Hkv, m, n], mu [Hkv, d]."""
    B, Hkv, S, d = K.shape
    I = S // n
    idx = np.unique(np.round(np.linspace(0, n - 1, m)).astype(np.int64))
    assert len(idx) == m
    theta = np.empty((Hkv, m, n))
    U = np.empty((Hkv, m, n))
    mu = np.empty((Hkv, d))
    for h in range(Hkv):
        Kb = K[:, h].reshape(B * I, n, d)
        Vb = V[:, h].reshape(B * I, n, d)
        mu[h] = Vb.mean(axis=(0, 1))
        Vc = np.concatenate(list(Vb - mu[h]), axis=1)              # [n, d * blocks]
        u, _, _ = np.linalg.svd(Vc, full_matrices=False)
        U[h] = u[:, :m].T
        Kc = np.concatenate(list(Kb), axis=1)                      # [n, d * blocks]
        theta[h] = (Kc @ np.linalg.pinv(Kc[idx])).T                # theta^T [n, m]
    return idx.astype(np.int32), theta, U, mu


def mean_cosine(a, b):
    """Mean over rows (last axis) of the cosine similarity."""
    num = (a * b).sum(-1)
    den = np.linalg.norm(a, axis=-1) * np.linalg.norm(b, axis=-1)
    return float((num / np.maximum(den, 1e-30)).mean())
