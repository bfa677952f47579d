"""ctypes front end of the KVCapsule CPU oracle (oracle/kvc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  It never imports the HIP package, and the HIP
package never imports it.  All arrays are host numpy float64, dense row-major;
the arithmetic lives entirely in the C file, this module only marshals.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvc_oracle.c")
_LIB = os.path.join(_HERE, "libkvc_oracle.so")

STORE_NONE = -1
STORE_F32 = 0
STORE_BF16 = 1

ACT_IDENTITY = 0
ACT_RELU = 1
ACT_GELU = 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.kvc_oracle_compressed_len.restype = ctypes.c_int32
        L.kvc_oracle_compressed_len.argtypes = [ctypes.c_int32, ctypes.c_double]
        L.kvc_oracle_round_to.restype = ctypes.c_double
        L.kvc_oracle_round_to.argtypes = [ctypes.c_double, ctypes.c_int]
        L.kvc_oracle_reconstruct_attend_decode.restype = ctypes.c_int
        L.kvc_oracle_num_threads.restype = ctypes.c_int
        L.kvc_oracle_static_attend_decode.restype = ctypes.c_int
        L.kvc_oracle_reconstruct_attend_decode_ragged.restype = ctypes.c_int
        _lib = L
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i32(x):
    return ctypes.c_int32(int(x))


def num_threads() -> int:
    return int(_load().kvc_oracle_num_threads())


def compressed_len(n: int, compression_ratio: float) -> int:
    return int(_load().kvc_oracle_compressed_len(int(n), float(compression_ratio)))


def round_to(x: float, store_dtype: int) -> float:
    return float(_load().kvc_oracle_round_to(float(x), int(store_dtype)))


def compress(K, V, key_idx, U, mu, n, I, vis_start, store_dtype=STORE_NONE):
    """K,V [B,Hkv,S,d]; key_idx [m]; U [Hkv,m,n]; mu [Hkv,d] -> Kc,Vc [B,Hkv,I,m,d]."""
    L = _load()
    K, pK = _d(K)
    V, pV = _d(V)
    U, pU = _d(U)
    mu, pmu = _d(mu)
    idx = np.ascontiguousarray(key_idx, dtype=np.int32)
    B, Hkv, S, d = K.shape
    m = idx.shape[0]
    assert V.shape == K.shape and U.shape == (Hkv, m, n) and mu.shape == (Hkv, d)
    assert 0 <= vis_start and vis_start + I * n <= S
    assert m == 0 or (idx.min() >= 0 and idx.max() < n)
    Kc = np.empty((B, Hkv, I, m, d), dtype=np.float64)
    Vc = np.empty((B, Hkv, I, m, d), dtype=np.float64)
    L.kvc_oracle_compress(_i32(B), _i32(Hkv), _i32(S), _i32(d), _i32(n), _i32(I), _i32(m),
                          _i32(vis_start), pK, pV, idx.ctypes.data_as(ctypes.c_void_p), pU, pmu,
                          ctypes.c_int(store_dtype), Kc.ctypes.data_as(ctypes.c_void_p),
                          Vc.ctypes.data_as(ctypes.c_void_p))
    return Kc, Vc


def reconstruct(Kc, Vc, theta, U, mu, n):
    """Kc,Vc [B,Hkv,I,m,d]; theta,U [Hkv,m,n]; mu [Hkv,d] -> Khat,Vhat [B,Hkv,I*n,d]."""
    L = _load()
    Kc, pKc = _d(Kc)
    Vc, pVc = _d(Vc)
    theta, pT = _d(theta)
    U, pU = _d(U)
    mu, pmu = _d(mu)
    B, Hkv, I, m, d = Kc.shape
    assert Vc.shape == Kc.shape and theta.shape == (Hkv, m, n) and U.shape == (Hkv, m, n)
    assert mu.shape == (Hkv, d)
    Khat = np.empty((B, Hkv, I * n, d), dtype=np.float64)
    Vhat = np.empty((B, Hkv, I * n, d), dtype=np.float64)
    L.kvc_oracle_reconstruct(_i32(B), _i32(Hkv), _i32(d), _i32(n), _i32(I), _i32(m), pKc, pVc, pT,
                             pU, pmu, Khat.ctypes.data_as(ctypes.c_void_p),
                             Vhat.ctypes.data_as(ctypes.c_void_p))
    return Khat, Vhat


def attend(q, Kvis, Vvis, Ktxt, Vtxt, t, scale=None, return_probs=False):
    """q [B,Hq,d]; Kvis,Vvis [B,Hkv,Nvis,d]; Ktxt,Vtxt [B,Hkv,Tcap,d] (first t rows valid).

    Returns out [B,Hq,d], lse [B,Hq] (and probs [B,Hq,Nvis+t])."""
    L = _load()
    q, pq = _d(q)
    Kvis, pKv = _d(Kvis)
    Vvis, pVv = _d(Vvis)
    B, Hq, d = q.shape
    Hkv, Nvis = Kvis.shape[1], Kvis.shape[2]
    assert Hq % Hkv == 0 and Kvis.shape == (B, Hkv, Nvis, d) and Vvis.shape == Kvis.shape
    if Ktxt is None:
        assert t == 0
        Tcap, pKt, pVt = 0, None, None
    else:
        Ktxt, pKt = _d(Ktxt)
        Vtxt, pVt = _d(Vtxt)
        Tcap = Ktxt.shape[2]
        assert Ktxt.shape == (B, Hkv, Tcap, d) and Vtxt.shape == Ktxt.shape and 0 <= t <= Tcap
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    probs = np.empty((B, Hq, Nvis + t), dtype=np.float64) if return_probs else None
    L.kvc_oracle_attend(_i32(B), _i32(Hq), _i32(Hkv), _i32(d), _i32(Nvis), pKv, pVv, _i32(t),
                        _i32(Tcap), pKt, pVt, pq, ctypes.c_double(scale),
                        out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p),
                        probs.ctypes.data_as(ctypes.c_void_p) if return_probs else None)
    return (out, lse, probs) if return_probs else (out, lse)


def attend_full(q, K, V, t, scale=None):
    """Full-cache ("All KV") attention of the paper's efficiency comparison: the attention equation
    of Sec. 3.1 over the first t rows of an uncompressed cache K, V [B,Hkv,cap,d].  This is
    kvc_oracle_attend with no vision rows; nothing is computed here."""
    K = np.asarray(K, dtype=np.float64)
    B, Hkv, _, d = K.shape
    none = np.zeros((B, Hkv, 0, d))
    return attend(q, none, none, K, V, t, scale)


def reconstruct_attend_decode(q, Kc, Vc, theta, U, mu, n, Ktxt, Vtxt, t, k_new=None, v_new=None,
                              scale=None):
    """One decode step of one layer.  Ktxt/Vtxt must be float64 C-contiguous arrays when
    k_new/v_new are given: the new token is written into them at row t (in place)."""
    L = _load()
    q, pq = _d(q)
    Kc, pKc = _d(Kc)
    Vc, pVc = _d(Vc)
    theta, pT = _d(theta)
    U, pU = _d(U)
    mu, pmu = _d(mu)
    B, Hq, d = q.shape
    _, Hkv, I, m, _ = Kc.shape
    assert Kc.shape == (B, Hkv, I, m, d) and Vc.shape == Kc.shape
    assert theta.shape == (Hkv, m, n) and U.shape == (Hkv, m, n) and mu.shape == (Hkv, d)
    if Ktxt is None:
        assert t == 0 and k_new is None
        Ktxt = np.zeros((B, Hkv, 1, d))
        Vtxt = np.zeros((B, Hkv, 1, d))
    if k_new is not None:
        assert Ktxt.dtype == np.float64 and Ktxt.flags.c_contiguous
        assert Vtxt.dtype == np.float64 and Vtxt.flags.c_contiguous
    Ktxt, pKt = _d(Ktxt)
    Vtxt, pVt = _d(Vtxt)
    Tcap = Ktxt.shape[2]
    assert Ktxt.shape == (B, Hkv, Tcap, d) and Vtxt.shape == Ktxt.shape
    pkn = pvn = None
    if k_new is not None:
        k_new, pkn = _d(k_new)
        v_new, pvn = _d(v_new)
        assert k_new.shape == (B, Hkv, d) and v_new.shape == (B, Hkv, d)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = L.kvc_oracle_reconstruct_attend_decode(
        _i32(B), _i32(Hq), _i32(Hkv), _i32(d), _i32(n), _i32(I), _i32(m), pKc, pVc, pT, pU, pmu,
        pKt, pVt, _i32(t), _i32(Tcap), pkn, pvn, pq, ctypes.c_double(scale),
        out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle decode failed (allocation, or append beyond capacity)")
    return out, lse


def mlp_hidden(Kc, W1, act, store_dtype=STORE_NONE):
    """First layer of the two-layer key reconstructor: Kc [B,Hkv,I,m,d], W1 [Hkv,m,m] -> H [B,Hkv,I,m,d]."""
    L = _load()
    Kc, pK = _d(Kc)
    W1, pW = _d(W1)
    B, Hkv, I, m, d = Kc.shape
    assert W1.shape == (Hkv, m, m)
    H = np.empty_like(Kc)
    L.kvc_oracle_mlp_hidden(_i32(B), _i32(Hkv), _i32(d), _i32(I), _i32(m), pK, pW, ctypes.c_int(act),
                            ctypes.c_int(store_dtype), H.ctypes.data_as(ctypes.c_void_p))
    return H


def static_attend_decode(q, Kc, Vc, Ktxt, Vtxt, t, k_new=None, v_new=None, scale=None):
    """Static variant (no reconstruction): attention over the compressed rows and the text cache."""
    L = _load()
    q, pq = _d(q)
    Kc, pKc = _d(Kc)
    Vc, pVc = _d(Vc)
    B, Hq, d = q.shape
    _, Hkv, I, m, _ = Kc.shape
    if Ktxt is None:
        assert t == 0 and k_new is None
        Ktxt = np.zeros((B, Hkv, 1, d))
        Vtxt = np.zeros((B, Hkv, 1, d))
    if k_new is not None:
        assert Ktxt.dtype == np.float64 and Ktxt.flags.c_contiguous
        assert Vtxt.dtype == np.float64 and Vtxt.flags.c_contiguous
    Ktxt, pKt = _d(Ktxt)
    Vtxt, pVt = _d(Vtxt)
    Tcap = Ktxt.shape[2]
    pkn = pvn = None
    if k_new is not None:
        k_new, pkn = _d(k_new)
        v_new, pvn = _d(v_new)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = L.kvc_oracle_static_attend_decode(_i32(B), _i32(Hq), _i32(Hkv), _i32(d), _i32(I), _i32(m), pKc, pVc,
                                           pKt, pVt, _i32(t), _i32(Tcap), pkn, pvn, pq, ctypes.c_double(scale),
                                           out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle static decode failed (append beyond capacity)")
    return out, lse


def reconstruct_attend_decode_ragged(q, Kc, Vc, theta, U, mu, n, n_images, text_len, Ktxt, Vtxt,
                                     k_new=None, v_new=None, scale=None):
    """Ragged decode step: n_images [B] (<= I), text_len [B]; Ktxt/Vtxt float64 C-contiguous, modified
    in place when k_new/v_new are given."""
    L = _load()
    q, pq = _d(q)
    Kc, pKc = _d(Kc)
    Vc, pVc = _d(Vc)
    theta, pT = _d(theta)
    U, pU = _d(U)
    mu, pmu = _d(mu)
    B, Hq, d = q.shape
    _, Hkv, I, m, _ = Kc.shape
    assert Ktxt.dtype == np.float64 and Ktxt.flags.c_contiguous and Vtxt.dtype == np.float64 and Vtxt.flags.c_contiguous
    Tcap = Ktxt.shape[2]
    ni = np.ascontiguousarray(n_images, dtype=np.int32)
    tl = np.ascontiguousarray(text_len, dtype=np.int32)
    assert ni.shape == (B,) and tl.shape == (B,)
    pkn = pvn = None
    if k_new is not None:
        k_new, pkn = _d(k_new)
        v_new, pvn = _d(v_new)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = L.kvc_oracle_reconstruct_attend_decode_ragged(
        _i32(B), _i32(Hq), _i32(Hkv), _i32(d), _i32(n), _i32(I), _i32(m), ni.ctypes.data_as(ctypes.c_void_p),
        tl.ctypes.data_as(ctypes.c_void_p), pKc, pVc, pT, pU, pmu, Ktxt.ctypes.data_as(ctypes.c_void_p),
        Vtxt.ctypes.data_as(ctypes.c_void_p), _i32(Tcap), pkn, pvn, pq, ctypes.c_double(scale),
        out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle ragged decode failed")
    return out, lse


def fused_order(q, Kc, Vc, theta, U, mu, n, Ktxt, Vtxt, t, scale=None):
    """Algorithm 1's evaluation order (joint softmax with text) -> out [B,Hq,d]."""
    L = _load()
    q, pq = _d(q)
    Kc, pKc = _d(Kc)
    Vc, pVc = _d(Vc)
    theta, pT = _d(theta)
    U, pU = _d(U)
    mu, pmu = _d(mu)
    B, Hq, d = q.shape
    _, Hkv, I, m, _ = Kc.shape
    if Ktxt is None:
        assert t == 0
        Ktxt = np.zeros((B, Hkv, 1, d))
        Vtxt = np.zeros((B, Hkv, 1, d))
    Ktxt, pKt = _d(Ktxt)
    Vtxt, pVt = _d(Vtxt)
    Tcap = Ktxt.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    L.kvc_oracle_fused_order(_i32(B), _i32(Hq), _i32(Hkv), _i32(d), _i32(n), _i32(I), _i32(m), pKc,
                             pVc, pT, pU, pmu, pKt, pVt, _i32(t), _i32(Tcap), pq,
                             ctypes.c_double(scale), out.ctypes.data_as(ctypes.c_void_p))
    return out


def memory_footprint(B, Hkv, c_prompt, n, I, m, t, d, b_kv, b_param):
    """App. C eqs. 1-2 in bytes -> (S_base, S_ours)."""
    L = _load()
    a = ctypes.c_int64()
    b = ctypes.c_int64()
    i64 = ctypes.c_int64
    L.kvc_oracle_memory_footprint(i64(B), i64(Hkv), i64(c_prompt), i64(n), i64(I), i64(m), i64(t),
                                  i64(d), i64(b_kv), i64(b_param), ctypes.byref(a), ctypes.byref(b))
    return int(a.value), int(b.value)
