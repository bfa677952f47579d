"""Fitted parameters on structured synthetic K/V (harness-side calibration, tests/calibration.py):
with redundancy of the kind Sec. 3.1 describes, compress + reconstruct recovers K and V and the
attention output stays close to full-cache attention.  The cosine similarities are the analogue of
what the paper's reconstruction-quality tables report; their values here belong to this synthetic
distribution only."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc

import calibration as cal

B, HKV, G, N, I, D, T = 2, 2, 2, 64, 3, 16, 5


def _full_attention(q, K, V, Kt, Vt, t):
    Hq = q.shape[1]
    Kf = np.concatenate([K, Kt[:, :, :t]], axis=2).repeat(Hq // K.shape[1], axis=1)
    Vf = np.concatenate([V, Vt[:, :, :t]], axis=2).repeat(Hq // K.shape[1], axis=1)
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[:, :, None, :], torch.from_numpy(Kf), torch.from_numpy(Vf))
    return out[:, :, 0].numpy()


def test_noiseless_rank_within_budget_is_exact():
    m, rank = 16, 12
    K, V, Ak, Av, mu0 = cal.make_structured_kv(1, B, HKV, N, I, D, rank, 0.0)
    idx, theta, U, mu = cal.fit_params(K, V, N, m)
    K2, V2, *_ = cal.make_structured_kv(2, B, HKV, N, I, D, rank, 0.0, Ak, Av, mu0)   # held out
    # the generating centre mu0 is used: with the fitted one, V2 - 1 mu^T would leave span(A) by the
    # direction 1 (mu0 - mu)^T
    Kc, Vc = orc.compress(K2, V2, idx, U, mu0, N, I, 0, orc.STORE_NONE)
    Kh, Vh = orc.reconstruct(Kc, Vc, theta, U, mu0, N)
    assert np.abs(Kh.reshape(K2.shape) - K2).max() < 1e-8
    assert np.abs(Vh.reshape(V2.shape) - V2).max() < 1e-8


@pytest.mark.parametrize("noise,floor", [(0.02, 0.995), (0.1, 0.93)])
def test_noisy_structured_data_reconstruction_quality(noise, floor):
    m, rank = 26, 12           # 60 % compression of n = 64
    assert orc.compressed_len(N, 0.6) == m
    K, V, Ak, Av, mu0 = cal.make_structured_kv(3, 6, HKV, N, I, D, rank, noise)
    idx, theta, U, mu = cal.fit_params(K, V, N, m)
    K2, V2, *_ = cal.make_structured_kv(4, B, HKV, N, I, D, rank, noise, Ak, Av, mu0)
    Kc, Vc = orc.compress(K2, V2, idx, U, mu, N, I, 0, orc.STORE_NONE)
    Kh, Vh = orc.reconstruct(Kc, Vc, theta, U, mu, N)
    ck = cal.mean_cosine(Kh.reshape(K2.shape), K2)
    cv = cal.mean_cosine(Vh.reshape(V2.shape), V2)
    print(f"[fitted] noise {noise}: cos(K_hat, K) = {ck:.4f}, cos(V_hat, V) = {cv:.4f}")
    assert ck >= floor and cv >= floor
    rng = np.random.default_rng(5)
    q = rng.standard_normal((B, HKV * G, D))
    Kt, Vt = rng.standard_normal((B, HKV, T, D)), rng.standard_normal((B, HKV, T, D))
    out, _ = orc.attend(q, Kh, Vh, Kt, Vt, T, None)
    ref = _full_attention(q, K2, V2, Kt, Vt, T)
    co = cal.mean_cosine(out, ref)
    print(f"[fitted] noise {noise}: cos(out, full-cache out) = {co:.4f}")
    assert co >= floor


def test_random_parameters_do_not_reconstruct():
    """Control: the quality above comes from the fit, not from the test."""
    m, rank = 26, 12
    K, V, Ak, Av, mu0 = cal.make_structured_kv(6, B, HKV, N, I, D, rank, 0.02)
    idx, theta, U, mu = cal.fit_params(K, V, N, m)
    rng = np.random.default_rng(7)
    theta_r = rng.standard_normal(theta.shape) / np.sqrt(m)
    Kc, Vc = orc.compress(K, V, idx, U, mu, N, I, 0, orc.STORE_NONE)
    Kh, _ = orc.reconstruct(Kc, Vc, theta_r, U, mu, N)
    assert cal.mean_cosine(Kh.reshape(K.shape), K) < 0.5
