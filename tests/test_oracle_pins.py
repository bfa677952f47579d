"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the HIP library.  Each test names the passage of the paper
(arxiv 2605.16439) or the textbook fact it pins the oracle to; the checks are
chosen so that a dropped term, a wrong sign or index, a transposed operand or a
swapped head mapping in oracle/kvc_oracle.c fails at least one of them.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import kvc_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def dct2_orthonormal(n):
    """Closed-form orthonormal DCT-II matrix (rows are basis vectors); not symmetric."""
    k = np.arange(n)[:, None]
    p = np.arange(n)[None, :]
    C = np.sqrt(2.0 / n) * np.cos(np.pi * (2 * p + 1) * k / (2.0 * n))
    C[0, :] *= np.sqrt(0.5)
    return C


def sdpa(q, K, V, scale):
    """Library attention (torch CPU, float64): q [B,Hq,d]; K,V [B,Hkv,X,d]."""
    q = torch.from_numpy(np.ascontiguousarray(q))[:, :, None, :]
    K = torch.from_numpy(np.ascontiguousarray(K))
    V = torch.from_numpy(np.ascontiguousarray(V))
    G = q.shape[1] // K.shape[1]
    K = K.repeat_interleave(G, dim=1)
    V = V.repeat_interleave(G, dim=1)
    return F.scaled_dot_product_attention(q, K, V, scale=scale)[:, :, 0, :].numpy()


# ---------------------------------------------------------------- compressed length
def test_compressed_len_golden():
    """|M_l| = ceil(l_r n) with l_r = 1 - c (Sec. 3.1, Keys); values in tests/golden."""
    rows = 0
    with open(os.path.join(GOLDEN, "compressed_len.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            n, c, m = line.split()
            assert orc.compressed_len(int(n), float(c)) == int(m), line
            rows += 1
    assert rows >= 10


def test_compressed_len_bounds():
    for n in (1, 7, 576, 1024):
        assert orc.compressed_len(n, 0.0) == n
        assert orc.compressed_len(n, 1.0) == 1          # at least one key is kept
        for c in np.linspace(0, 1, 41):
            m = orc.compressed_len(n, float(c))
            assert 1 <= m <= n
            assert m >= (1 - c) * n - 1e-6 and m < (1 - c) * n + 1 + 1e-6 or m == 1


# ---------------------------------------------------------------- storage rounding
def test_round_bf16_matches_library_and_ties():
    x = rng(1).standard_normal(4000).astype(np.float32) * np.float32(37.0)
    x = np.concatenate([x, np.float32([1e-30, -3e-39, 6.5e4, 3.0e38, 0.0])])
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([orc.round_to(float(v), orc.STORE_BF16) for v in x])
    assert np.array_equal(lib, got)
    # ties go to the even significand: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert orc.round_to(1.0 + 2.0 ** -8, orc.STORE_BF16) == 1.0
    assert orc.round_to(1.0 + 3 * 2.0 ** -8, orc.STORE_BF16) == 1.0 + 2.0 ** -6
    assert orc.round_to(1.0 + 2.0 ** -8 + 2.0 ** -30, orc.STORE_BF16) == 1.0 + 2.0 ** -7
    assert orc.round_to(0.1, orc.STORE_F32) == float(np.float32(0.1))
    assert orc.round_to(0.1, orc.STORE_NONE) == 0.1


# ---------------------------------------------------------------- ratio 0 reproduces input
def test_ratio_zero_reproduces_input():
    """m = n, M = identity, theta = I, U orthonormal: K_hat = K exactly and V_hat = V
    (Sec. 3.1: V_tilde = U(V - 1 mu^T), V_hat = U^T V_tilde + 1 mu^T) for any mu."""
    r = rng(2)
    B, Hkv, d, n, I, pre, post = 2, 2, 8, 12, 3, 2, 3
    S = pre + I * n + post
    K = r.standard_normal((B, Hkv, S, d))
    V = r.standard_normal((B, Hkv, S, d))
    U = np.stack([dct2_orthonormal(n), dct2_orthonormal(n)[::-1].copy()])
    theta = np.stack([np.eye(n)] * Hkv)
    mu = r.standard_normal((Hkv, d))
    idx = np.arange(n, dtype=np.int32)
    Kc, Vc = orc.compress(K, V, idx, U, mu, n, I, pre)
    assert np.array_equal(Kc.reshape(B, Hkv, I * n, d), K[:, :, pre:pre + I * n])
    Khat, Vhat = orc.reconstruct(Kc, Vc, theta, U, mu, n)
    assert np.array_equal(Khat, K[:, :, pre:pre + I * n])
    assert np.abs(Vhat - V[:, :, pre:pre + I * n]).max() < 1e-12


def test_key_rows_are_selected_in_mask_order():
    """K_tilde is the row selection K[M] (Sec. 3.1), per image block, heads share M."""
    r = rng(3)
    B, Hkv, d, n, I, pre = 1, 3, 4, 9, 2, 5
    S = pre + I * n + 1
    K = r.standard_normal((B, Hkv, S, d))
    V = r.standard_normal((B, Hkv, S, d))
    idx = np.array([1, 4, 5, 8], dtype=np.int32)
    m = len(idx)
    U = r.standard_normal((Hkv, m, n))
    mu = r.standard_normal((Hkv, d))
    Kc, Vc = orc.compress(K, V, idx, U, mu, n, I, pre)
    for i in range(I):
        assert np.array_equal(Kc[:, :, i], K[:, :, pre + i * n + idx])
    # values: centred projection, per head, checked with a library matmul
    for h in range(Hkv):
        for i in range(I):
            Z = V[0, h, pre + i * n: pre + (i + 1) * n] - mu[h][None, :]
            assert np.allclose(Vc[0, h, i], U[h] @ Z, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- values: PCA closed forms
def test_value_path_low_rank_exact_and_eckart_young():
    """U from an SVD of centred values (Sec. 3.1): rank <= m is recovered exactly; for
    higher rank the residual equals sqrt(sum of the discarded singular values^2)."""
    r = rng(4)
    n, d, m = 16, 6, 4
    mu = r.standard_normal((1, d))
    # rank-3 centred values
    Zc = r.standard_normal((n, 3)) @ r.standard_normal((3, d))
    V = (Zc + mu)[None, None]
    Uf, s, _ = np.linalg.svd(Zc, full_matrices=False)
    U = Uf[:, :m].T[None]                         # [1, m, n], orthonormal rows
    K = r.standard_normal(V.shape)
    idx = np.arange(m, dtype=np.int32)
    Kc, Vc = orc.compress(K, V, idx, U, mu, n, 1, 0)
    _, Vhat = orc.reconstruct(Kc, Vc, np.zeros((1, m, n)), U, mu, n)
    assert np.abs(Vhat - V).max() < 1e-12
    # full-rank values: Frobenius error of the best rank-m approximation
    Zc = r.standard_normal((n, d))
    V = (Zc + mu)[None, None]
    Uf, s, _ = np.linalg.svd(Zc, full_matrices=False)
    U = Uf[:, :m].T[None]
    Kc, Vc = orc.compress(K, V, idx, U, mu, n, 1, 0)
    _, Vhat = orc.reconstruct(Kc, Vc, np.zeros((1, m, n)), U, mu, n)
    err = np.linalg.norm(Vhat[0, 0] - V[0, 0])
    assert abs(err - np.sqrt((s[m:] ** 2).sum())) < 1e-12


# ---------------------------------------------------------------- keys: recoverable case
def test_recoverable_keys_equal_full_cache_attention():
    """If K = C K_tilde with C the identity on retained rows and theta = C^T, then
    K_hat = K; with orthonormal square U the values are exact too, so the decode
    output must equal library attention over the uncompressed cache (Sec. 3.2)."""
    r = rng(5)
    B, Hq, Hkv, d, n, I, t = 2, 6, 2, 8, 10, 2, 5
    m = 4
    idx = np.array([0, 3, 6, 9], dtype=np.int32)
    C = r.standard_normal((Hkv, n, m)) * 0.5
    for h in range(Hkv):
        C[h, idx, :] = np.eye(m)
    Kt = r.standard_normal((B, Hkv, I, m, d))
    K = np.einsum("hpm,bhimd->bhipd", C, Kt).reshape(B, Hkv, I * n, d)
    theta = np.ascontiguousarray(C.transpose(0, 2, 1))          # [Hkv, m, n]
    V = r.standard_normal((B, Hkv, I * n, d))
    Ktxt = r.standard_normal((B, Hkv, t + 2, d))
    Vtxt = r.standard_normal((B, Hkv, t + 2, d))
    q = r.standard_normal((B, Hq, d))
    mu = r.standard_normal((Hkv, d))
    # keys through the compressed path (m < n), values through a square orthonormal U
    Kc, _ = orc.compress(K, V, idx, np.zeros((Hkv, m, n)), mu, n, I, 0)
    assert np.array_equal(Kc, Kt)
    Khat, _ = orc.reconstruct(Kc, Kc, theta, np.zeros((Hkv, m, n)), mu, n)
    assert np.abs(Khat - K).max() < 1e-12
    Un = np.stack([dct2_orthonormal(n)] * Hkv)
    _, Vc = orc.compress(K, V, np.arange(n, dtype=np.int32), Un, mu, n, I, 0)
    _, Vhat = orc.reconstruct(Vc, Vc, Un, Un, mu, n)
    out, lse = orc.attend(q, Khat, Vhat, Ktxt, Vtxt, t)
    ref = sdpa(q, np.concatenate([K, Ktxt[:, :, :t]], 2), np.concatenate([V, Vtxt[:, :, :t]], 2),
               1.0 / np.sqrt(d))
    assert np.abs(out - ref).max() < 1e-12


# ---------------------------------------------------------------- attention invariants
def _tiny_problem(seed, B=2, Hq=4, Hkv=2, d=8, n=12, I=2, m=5, t=3, cap=5):
    r = rng(seed)
    p = dict(B=B, Hq=Hq, Hkv=Hkv, d=d, n=n, I=I, m=m, t=t)
    p["Kc"] = r.standard_normal((B, Hkv, I, m, d))
    p["Vc"] = r.standard_normal((B, Hkv, I, m, d))
    p["theta"] = r.standard_normal((Hkv, m, n)) / np.sqrt(m)
    p["U"] = r.standard_normal((Hkv, m, n)) / np.sqrt(n)
    p["mu"] = r.standard_normal((Hkv, d))
    p["Ktxt"] = r.standard_normal((B, Hkv, cap, d))
    p["Vtxt"] = r.standard_normal((B, Hkv, cap, d))
    p["q"] = r.standard_normal((B, Hq, d))
    return p


def test_attention_probabilities_and_mean():
    p = _tiny_problem(6)
    Khat, Vhat = orc.reconstruct(p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], p["n"])
    out, lse, probs = orc.attend(p["q"], Khat, Vhat, p["Ktxt"], p["Vtxt"], p["t"],
                                 return_probs=True)
    assert probs.shape[-1] == p["I"] * p["n"] + p["t"]
    assert np.all(probs > 0) and np.abs(probs.sum(-1) - 1).max() < 1e-14
    # q = 0: uniform weights -> mean of all N + t value rows of the head's KV group
    out0, lse0 = orc.attend(np.zeros_like(p["q"]), Khat, Vhat, p["Ktxt"], p["Vtxt"], p["t"])
    allV = np.concatenate([Vhat, p["Vtxt"][:, :, :p["t"]]], 2)
    G = p["Hq"] // p["Hkv"]
    for g in range(p["Hq"]):
        assert np.abs(out0[:, g] - allV[:, g // G].mean(1)).max() < 1e-13
    assert np.abs(lse0 - np.log(allV.shape[2])).max() < 1e-13
    # lse is the log of the softmax denominator
    s = np.einsum("bgd,bgxd->bgx", p["q"], np.concatenate(
        [Khat, p["Ktxt"][:, :, :p["t"]]], 2).repeat(G, axis=1)) / np.sqrt(p["d"])
    assert np.abs(lse - np.log(np.exp(s).sum(-1))).max() < 1e-12


def test_attention_sharp_limit_selects_argmax_row():
    p = _tiny_problem(7)
    Khat, Vhat = orc.reconstruct(p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], p["n"])
    out, _ = orc.attend(p["q"], Khat, Vhat, p["Ktxt"], p["Vtxt"], p["t"], scale=1e4)
    allK = np.concatenate([Khat, p["Ktxt"][:, :, :p["t"]]], 2)
    allV = np.concatenate([Vhat, p["Vtxt"][:, :, :p["t"]]], 2)
    G = p["Hq"] // p["Hkv"]
    for b in range(p["B"]):
        for g in range(p["Hq"]):
            x = np.argmax(allK[b, g // G] @ p["q"][b, g])
            assert np.abs(out[b, g] - allV[b, g // G, x]).max() < 1e-9


def test_gqa_mapping_and_block_permutation():
    p = _tiny_problem(8)
    # query heads of one group with equal q give equal outputs; different groups differ
    q = p["q"].copy()
    q[:, 1] = q[:, 0]
    q[:, 2] = q[:, 0]
    out, _ = orc.reconstruct_attend_decode(q, p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                           p["n"], p["Ktxt"], p["Vtxt"], p["t"])
    assert np.array_equal(out[:, 0], out[:, 1])          # heads 0,1 -> KV head 0
    assert np.abs(out[:, 0] - out[:, 2]).max() > 1e-3    # head 2 -> KV head 1
    # softmax over a set: permuting the image blocks of the capsule changes nothing
    perm = [1, 0]
    out2, _ = orc.reconstruct_attend_decode(q, p["Kc"][:, :, perm], p["Vc"][:, :, perm],
                                            p["theta"], p["U"], p["mu"], p["n"], p["Ktxt"],
                                            p["Vtxt"], p["t"])
    assert np.abs(out - out2).max() < 1e-13
    # rows of the text cache beyond t are ignored
    Kt2 = p["Ktxt"].copy()
    Kt2[:, :, p["t"]:] = 1e3
    out3, _ = orc.reconstruct_attend_decode(q, p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                            p["n"], Kt2, p["Vtxt"], p["t"])
    assert np.array_equal(out, out3)


# ---------------------------------------------------------------- library attention
def test_text_only_is_plain_sdpa():
    p = _tiny_problem(9, I=0, t=5, cap=5)
    out, _ = orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                           p["n"], p["Ktxt"], p["Vtxt"], 5, scale=0.3)
    assert np.abs(out - sdpa(p["q"], p["Ktxt"], p["Vtxt"], 0.3)).max() < 1e-13


def test_full_cache_attention_is_library_sdpa_on_the_concatenation():
    """The "All KV" comparison point (Sec. 4 / Fig. 5): attention over [K_vis ; K_txt] with nothing
    compressed.  Both ways of handing the rows to the oracle (two buffers, or one full cache) equal
    the library's attention on the concatenated rows, GQA included; rows beyond t are ignored."""
    r = rng(41)
    B, Hq, Hkv, d, N, t, cap = 2, 6, 2, 8, 11, 5, 8
    q = r.standard_normal((B, Hq, d))
    Kv, Vv = r.standard_normal((B, Hkv, N, d)), r.standard_normal((B, Hkv, N, d))
    Kt, Vt = r.standard_normal((B, Hkv, cap, d)), r.standard_normal((B, Hkv, cap, d))
    scale = 0.41
    Kall = np.concatenate([Kv, Kt[:, :, :t]], 2)
    Vall = np.concatenate([Vv, Vt[:, :, :t]], 2)
    ref = sdpa(q, Kall, Vall, scale)
    out, lse = orc.attend(q, Kv, Vv, Kt, Vt, t, scale)
    assert np.abs(out - ref).max() < 1e-13
    pad = r.standard_normal((B, Hkv, 3, d)) * 50.0                  # garbage beyond the valid rows
    out2, lse2 = orc.attend_full(q, np.concatenate([Kall, pad], 2), np.concatenate([Vall, pad], 2), N + t, scale)
    assert np.abs(out2 - ref).max() < 1e-13
    assert np.abs(lse2 - lse).max() < 1e-13
    G = Hq // Hkv
    s = scale * np.einsum("bgd,bgxd->bgx", q, Kall.repeat(G, axis=1))
    assert np.abs(lse2 - np.log(np.exp(s).sum(-1))).max() < 1e-12


def test_block_diagonal_dense_form_matches_library():
    """Independent construction: per-block reconstruction written as one dense
    block-diagonal matrix (kron), then library matmul + library SDPA."""
    p = _tiny_problem(10, Hq=6, Hkv=3, n=7, I=3, m=4, t=4, cap=4)
    B, Hkv, I, m, n, d = p["B"], p["Hkv"], p["I"], p["m"], p["n"], p["d"]
    Kfull = np.empty((B, Hkv, I * n, d))
    Vfull = np.empty((B, Hkv, I * n, d))
    for h in range(Hkv):
        RK = np.kron(np.eye(I), p["theta"][h].T)             # [I n, I m]
        RV = np.kron(np.eye(I), p["U"][h].T)
        for b in range(B):
            Kfull[b, h] = RK @ p["Kc"][b, h].reshape(I * m, d)
            Vfull[b, h] = RV @ p["Vc"][b, h].reshape(I * m, d) + p["mu"][h][None]
    ref = sdpa(p["q"], np.concatenate([Kfull, p["Ktxt"]], 2),
               np.concatenate([Vfull, p["Vtxt"]], 2), 1.0 / np.sqrt(d))
    out, _ = orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                           n, p["Ktxt"], p["Vtxt"], 4)
    assert np.abs(out - ref).max() < 1e-12


# ---------------------------------------------------------------- Algorithm 1 equivalence
@pytest.mark.parametrize("t", [0, 3])
def test_algorithm1_order_equals_reconstruct_then_attend(t):
    """Alg. 1 (score-space order, associativity of Sec. 4 efficiency analysis) gives the
    same result as reconstruct-then-attend; GQA and text tokens included."""
    p = _tiny_problem(11 + t, t=t)
    a, _ = orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                         p["n"], p["Ktxt"], p["Vtxt"], t)
    b = orc.fused_order(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], p["n"],
                        p["Ktxt"], p["Vtxt"], t)
    assert np.abs(a - b).max() < 1e-10


# ---------------------------------------------------------------- decode step semantics
def test_append_new_token_then_attend():
    p = _tiny_problem(12, t=3, cap=5)
    r = rng(13)
    kn = r.standard_normal((p["B"], p["Hkv"], p["d"]))
    vn = r.standard_normal((p["B"], p["Hkv"], p["d"]))
    Kt = p["Ktxt"].copy()
    Vt = p["Vtxt"].copy()
    out, _ = orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                           p["n"], Kt, Vt, 3, k_new=kn, v_new=vn)
    assert np.array_equal(Kt[:, :, 3], kn) and np.array_equal(Vt[:, :, 3], vn)
    assert np.array_equal(Kt[:, :, :3], p["Ktxt"][:, :, :3])
    ref, _ = orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                           p["n"], Kt, Vt, 4)
    assert np.array_equal(out, ref)
    with pytest.raises(RuntimeError):
        orc.reconstruct_attend_decode(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"],
                                      p["n"], Kt, Vt, 5, k_new=kn, v_new=vn)


# ---------------------------------------------------------------- memory model
def test_memory_footprint_closed_form():
    """App. C eqs. 1-2, hand-evaluated: B=1, H_kv=4, c=0, one image n=1024, m=410, t=0,
    d=128, 2-byte elements."""
    base, ours = orc.memory_footprint(1, 4, 0, 1024, 1, 410, 0, 128, 2, 2)
    assert base == 2 * 4 * 1024 * 128 * 2 == 2097152
    # KV 2*4*410*128*2 = 839680; theta and U 4*410*1024*2 = 3358720 each; mu 4*128*2 = 1024
    assert ours == 839680 + 3358720 + 3358720 + 1024 == 7558144
    # prompt and generated tokens enter both sides equally
    b2, o2 = orc.memory_footprint(3, 4, 100, 1024, 8, 410, 50, 128, 2, 2)
    assert b2 - o2 == 3 * (2 * 4 * 8 * (1024 - 410) * 128 * 2) - (2 * 3358720 + 1024)


def test_capsule_size_matches_ratio():
    """Stored vision length drops from n to ceil(l_r n) (App. C): capsule bytes / vision
    KV bytes = m / n at the benchmark shapes."""
    for n, c in ((576, 0.6), (1024, 0.6), (1024, 0.4), (1024, 0.8), (256, 0.6)):
        m = orc.compressed_len(n, c)
        r = rng(n)
        K = r.standard_normal((1, 1, n, 2))
        idx = np.sort(r.choice(n, m, replace=False)).astype(np.int32)
        Kc, Vc = orc.compress(K, K, idx, np.zeros((1, m, n)), np.zeros((1, 2)), n, 1, 0)
        assert (Kc.size + Vc.size) / (2.0 * K.size) == m / n
        assert abs(m / n - (1 - c)) < 1.0 / n


# ---------------------------------------------------------------- brute force on a tiny case
def test_brute_force_python_loops_on_tiny_case():
    """Sec. 3.1 / 3.2 written out a second time as scalar Python loops (no matrix routines):
    compress, reconstruct, joint softmax over vision and text, GQA, new-token append."""
    import math
    B, Hq, Hkv, d, n, I, m, t = 2, 4, 2, 3, 5, 2, 3, 2
    G = Hq // Hkv
    r = rng(77)
    K = r.standard_normal((B, Hkv, 1 + I * n + 1, d))        # one row before and after the span
    V = r.standard_normal((B, Hkv, 1 + I * n + 1, d))
    idx = np.array([0, 2, 4], dtype=np.int32)
    theta = r.standard_normal((Hkv, m, n))
    U = r.standard_normal((Hkv, m, n))
    mu = r.standard_normal((Hkv, d))
    q = r.standard_normal((B, Hq, d))
    Kt = r.standard_normal((B, Hkv, t + 1, d))
    Vt = r.standard_normal((B, Hkv, t + 1, d))
    kn, vn = r.standard_normal((B, Hkv, d)), r.standard_normal((B, Hkv, d))
    scale = 0.7

    Kc, Vc = orc.compress(K, V, idx, U, mu, n, I, 1)
    out, lse = orc.reconstruct_attend_decode(q, Kc, Vc, theta, U, mu, n, Kt.copy(), Vt.copy(), t, kn, vn,
                                             scale)
    for b in range(B):
        for gq in range(Hq):
            h = gq // G
            keys, vals = [], []
            for i in range(I):
                # capsule of block i
                kc = [[K[b, h, 1 + i * n + idx[j], c] for c in range(d)] for j in range(m)]
                vc = [[sum(U[h, j, p] * (V[b, h, 1 + i * n + p, c] - mu[h, c]) for p in range(n))
                       for c in range(d)] for j in range(m)]
                for p in range(n):
                    keys.append([sum(theta[h, j, p] * kc[j][c] for j in range(m)) for c in range(d)])
                    vals.append([sum(U[h, j, p] * vc[j][c] for j in range(m)) + mu[h, c] for c in range(d)])
            for x in range(t):
                keys.append(list(Kt[b, h, x]))
                vals.append(list(Vt[b, h, x]))
            keys.append(list(kn[b, h]))
            vals.append(list(vn[b, h]))
            logits = [scale * sum(q[b, gq, c] * k[c] for c in range(d)) for k in keys]
            mx = max(logits)
            w = [math.exp(s - mx) for s in logits]
            z = sum(w)
            for c in range(d):
                y = sum(w[x] * vals[x][c] for x in range(len(vals))) / z
                assert abs(out[b, gq, c] - y) < 1e-12
            assert abs(lse[b, gq] - (mx + math.log(z))) < 1e-12


# ---------------------------------------------------------------- storage rounding inside compress
def test_compress_with_bf16_storage_is_one_rounding_of_the_exact_result():
    """Sec. 3.1 (Values) gives V_tilde exactly; the stored capsule is that value rounded ONCE to
    the storage type.  The oracle's compress with a storage type must therefore equal the library's
    (torch) bf16 / fp32 rounding of its own unrounded result, and the keys must stay exact copies."""
    r = rng(21)
    B, Hkv, d, n, I, pre = 2, 2, 16, 24, 2, 3
    S = pre + I * n + 2
    K = torch.from_numpy(r.standard_normal((B, Hkv, S, d))).to(torch.bfloat16).to(torch.float64).numpy()
    V = r.standard_normal((B, Hkv, S, d)) * 3.0
    idx = np.array([0, 2, 3, 7, 11, 12, 19, 23], dtype=np.int32)
    m = len(idx)
    U = r.standard_normal((Hkv, m, n))
    mu = r.standard_normal((Hkv, d))
    Kc0, Vc0 = orc.compress(K, V, idx, U, mu, n, I, pre, orc.STORE_NONE)
    Kc1, Vc1 = orc.compress(K, V, idx, U, mu, n, I, pre, orc.STORE_BF16)
    Kc2, Vc2 = orc.compress(K, V, idx, U, mu, n, I, pre, orc.STORE_F32)
    assert np.array_equal(Kc0, Kc1) and np.array_equal(Kc0, Kc2)
    # double -> float -> bfloat16 would round twice; the exact double is rounded directly here
    # (values whose double lies within 2^-24 of a bf16 tie are not in this sample: checked below)
    lib_bf16 = torch.from_numpy(Vc0).to(torch.bfloat16).to(torch.float64).numpy()
    lib_f32 = Vc0.astype(np.float32).astype(np.float64)
    assert np.array_equal(Vc2, lib_f32)
    differs = Vc1 != lib_bf16
    if differs.any():       # only where float32 rounding moved the value onto a bf16 tie
        x = Vc0[differs]
        assert np.all(np.abs(x.astype(np.float32).astype(np.float64) - x) > 0)
        assert differs.sum() <= 2
    # one rounding: the error is at most half a unit in the last place of bf16 (8 significand bits)
    nz = Vc0 != 0
    assert np.all(np.abs(Vc1[nz] - Vc0[nz]) <= np.abs(Vc0[nz]) * 2.0 ** -8)
    assert np.abs(Vc1 - Vc0).max() > 0


# ---------------------------------------------------------------- softmax shift invariance
def test_attention_is_invariant_to_a_common_logit_shift_and_survives_large_logits():
    """softmax(s + c) = softmax(s) (Sec. 3.1, attention equation).  A common shift of all logits
    is produced exactly by one extra key channel that is constant over all keys: the output must
    not move and lse must move by the shift, also when the shifted logits (+-800) would overflow
    or underflow exp() without the subtraction of the maximum."""
    p = _tiny_problem(31)
    Khat, Vhat = orc.reconstruct(p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], p["n"])
    B, Hkv, d = p["B"], p["Hkv"], p["d"]
    t = p["t"]
    out, lse = orc.attend(p["q"], Khat, Vhat, p["Ktxt"], p["Vtxt"], t, scale=1.0)
    ones_v = np.ones(Khat.shape[:-1] + (1,))
    ones_t = np.ones(p["Ktxt"].shape[:-1] + (1,))
    zeros_v = np.zeros(Vhat.shape[:-1] + (1,))
    zeros_t = np.zeros(p["Vtxt"].shape[:-1] + (1,))
    for shift in (3.5, 800.0, -800.0):
        q2 = np.concatenate([p["q"], np.full(p["q"].shape[:-1] + (1,), shift)], -1)
        out2, lse2 = orc.attend(q2, np.concatenate([Khat, ones_v], -1), np.concatenate([Vhat, zeros_v], -1),
                                np.concatenate([p["Ktxt"], ones_t], -1), np.concatenate([p["Vtxt"], zeros_t], -1),
                                t, scale=1.0)
        assert np.all(np.isfinite(out2)) and np.all(np.isfinite(lse2))
        assert np.abs(out2[..., :d] - out).max() < 1e-12
        assert np.abs(out2[..., d]).max() == 0.0
        assert np.abs(lse2 - (lse + shift)).max() < 1e-10
    # large spread: logits of +-1000 around the maximum; the winner takes all, nothing is NaN
    q3 = p["q"] * 300.0
    out3, lse3 = orc.attend(q3, Khat, Vhat, p["Ktxt"], p["Vtxt"], t, scale=1.0)
    assert np.all(np.isfinite(out3)) and np.all(np.isfinite(lse3))
    allK = np.concatenate([Khat, p["Ktxt"][:, :, :t]], 2)
    G = p["Hq"] // Hkv
    for b in range(B):
        for g in range(p["Hq"]):
            s = allK[b, g // G] @ q3[b, g]
            assert abs(lse3[b, g] - (s.max() + np.log(np.exp(s - s.max()).sum()))) < 1e-9


# ---------------------------------------------------------------- two-layer key reconstructor
def test_two_layer_reconstructor_collapses_to_the_linear_one_and_matches_library_ops():
    """Sec. 3.1 (Keys): f_theta as a two-layer MLP along the sequence axis.  With the identity between
    the layers it is the linear reconstruction with theta = W1 W2 (App. C's score reconstruction matrix);
    with ReLU / GELU the first layer equals the library's matmul + activation; keys that the first layer
    leaves positive pass ReLU unchanged."""
    r = rng(51)
    B, Hkv, d, n, I, m = 2, 2, 6, 11, 2, 4
    Kc = r.standard_normal((B, Hkv, I, m, d))
    W1 = r.standard_normal((Hkv, m, m))
    W2 = r.standard_normal((Hkv, m, n))
    zeroU, mu = np.zeros((Hkv, m, n)), np.zeros((Hkv, d))
    H0 = orc.mlp_hidden(Kc, W1, orc.ACT_IDENTITY)
    Khat2, _ = orc.reconstruct(H0, H0, W2, zeroU, mu, n)
    theta = np.einsum("hjr,hrp->hjp", W1, W2)
    Khat1, _ = orc.reconstruct(Kc, Kc, theta, zeroU, mu, n)
    assert np.abs(Khat2 - Khat1).max() < 1e-12
    lin = torch.einsum("hjr,bhijd->bhird", torch.from_numpy(W1), torch.from_numpy(Kc))
    assert np.abs(orc.mlp_hidden(Kc, W1, orc.ACT_RELU) - F.relu(lin).numpy()).max() < 1e-13
    assert np.abs(orc.mlp_hidden(Kc, W1, orc.ACT_GELU) - F.gelu(lin).numpy()).max() < 1e-12
    assert np.any(lin.numpy() < 0)
    Kpos, Wpos = np.abs(Kc), np.abs(W1)
    assert np.array_equal(orc.mlp_hidden(Kpos, Wpos, orc.ACT_RELU), orc.mlp_hidden(Kpos, Wpos, orc.ACT_IDENTITY))
    # stored form: one rounding of the exact value
    Hb = orc.mlp_hidden(Kc, W1, orc.ACT_GELU, orc.STORE_BF16)
    Hx = orc.mlp_hidden(Kc, W1, orc.ACT_GELU)
    assert np.all(np.abs(Hb - Hx) <= np.abs(Hx) * 2.0 ** -8 + 1e-300) and np.abs(Hb - Hx).max() > 0
    # transposed W1 must not pass: the first layer contracts the ROW index of W1 with the key rows
    assert np.abs(orc.mlp_hidden(Kc, np.ascontiguousarray(W1.transpose(0, 2, 1)), orc.ACT_RELU) - F.relu(lin).numpy()).max() > 1e-3


# ---------------------------------------------------------------- static variant
def test_static_variant_is_library_attention_over_the_compressed_rows():
    """Ablation appendix (static compression without reconstruction): the compressed KV is used directly,
    i.e. plain attention over the I*m compressed rows and the text rows, new token appended first."""
    p = _tiny_problem(52)
    B, Hkv, d, I, m, t = p["B"], p["Hkv"], p["d"], p["I"], p["m"], p["t"]
    r = rng(53)
    kn, vn = r.standard_normal((B, Hkv, d)), r.standard_normal((B, Hkv, d))
    Kt, Vt = p["Ktxt"].copy(), p["Vtxt"].copy()
    out, lse = orc.static_attend_decode(p["q"], p["Kc"], p["Vc"], Kt, Vt, t, kn, vn, scale=0.3)
    assert np.array_equal(Kt[:, :, t], kn) and np.array_equal(Vt[:, :, t], vn)
    Kall = np.concatenate([p["Kc"].reshape(B, Hkv, I * m, d), p["Ktxt"][:, :, :t], kn[:, :, None]], 2)
    Vall = np.concatenate([p["Vc"].reshape(B, Hkv, I * m, d), p["Vtxt"][:, :, :t], vn[:, :, None]], 2)
    assert np.abs(out - sdpa(p["q"], Kall, Vall, 0.3)).max() < 1e-13
    # m = n with identity parameters and mu = 0: reconstruction changes nothing, both variants agree
    n = p["n"]
    Kc, Vc = rng(54).standard_normal((B, Hkv, I, n, d)), rng(55).standard_normal((B, Hkv, I, n, d))
    eye = np.stack([np.eye(n)] * Hkv)
    a, _ = orc.static_attend_decode(p["q"], Kc, Vc, p["Ktxt"], p["Vtxt"], t)
    b, _ = orc.reconstruct_attend_decode(p["q"], Kc, Vc, eye, eye, np.zeros((Hkv, d)), n, p["Ktxt"], p["Vtxt"], t)
    assert np.abs(a - b).max() < 1e-13


# ---------------------------------------------------------------- ragged batch
def test_ragged_batch_equals_the_sequences_taken_one_by_one():
    p = _tiny_problem(56, B=4, I=3, cap=7)
    B, Hkv, d, n = p["B"], p["Hkv"], p["d"], p["n"]
    r = rng(57)
    kn, vn = r.standard_normal((B, Hkv, d)), r.standard_normal((B, Hkv, d))
    n_images, text_len = [3, 0, 1, 2], [2, 5, 0, 6]
    Kt, Vt = p["Ktxt"].copy(), p["Vtxt"].copy()
    out, lse = orc.reconstruct_attend_decode_ragged(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], n,
                                                    n_images, text_len, Kt, Vt, kn, vn)
    for b in range(B):
        Ib, tb = n_images[b], text_len[b]
        Kb, Vb = p["Ktxt"][b:b + 1].copy(), p["Vtxt"][b:b + 1].copy()
        ref, lref = orc.reconstruct_attend_decode(p["q"][b:b + 1], p["Kc"][b:b + 1, :, :Ib], p["Vc"][b:b + 1, :, :Ib],
                                                  p["theta"], p["U"], p["mu"], n, Kb, Vb, tb, kn[b:b + 1], vn[b:b + 1])
        assert np.array_equal(out[b], ref[0]) and np.array_equal(lse[b], lref[0])
        assert np.array_equal(Kt[b], Kb[0]) and np.array_equal(Vt[b], Vb[0])
        # blocks beyond the sequence's count and text rows beyond its length do not matter
    Kc2 = p["Kc"].copy()
    Kc2[1] = 1e3
    Kc2[2, :, 1:] = -1e3
    out2, _ = orc.reconstruct_attend_decode_ragged(p["q"], Kc2, p["Vc"], p["theta"], p["U"], p["mu"], n, n_images,
                                                   text_len, p["Ktxt"].copy(), p["Vtxt"].copy(), kn, vn)
    assert np.array_equal(out, out2)
    with pytest.raises(RuntimeError):
        orc.reconstruct_attend_decode_ragged(p["q"], p["Kc"], p["Vc"], p["theta"], p["U"], p["mu"], n, [4, 0, 0, 0],
                                             text_len, p["Ktxt"].copy(), p["Vtxt"].copy())
