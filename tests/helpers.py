"""Shared plumbing of the tests: run the oracle / the HIP library on the same seeded
tensors and measure the error.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2605_16439_amd import synth


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def store_code(w: synth.Workload) -> int:
    from oracle import kvc_oracle as orc
    return orc.STORE_F32 if w.dtype == "f32" else orc.STORE_BF16


def tol(w: synth.Workload) -> float:
    """Relative-error bar on the attention output: 1e-5 for fp32, 2e-2 for bf16."""
    return 1e-5 if w.dtype == "f32" else 2e-2


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over leading rows of ||got - ref||_2 / ||ref||_2 (last axis)."""
    num = np.linalg.norm(got - ref, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


def elem_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over all elements of |got - ref| / rms(ref row): the element-wise companion of
    row_rel_err (one channel of a row cannot hide behind the row's norm)."""
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    return float((np.abs(got - ref) / np.maximum(rms, 1e-30)).max())


def block_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over (b, h, i) blocks of the Frobenius-norm relative error."""
    num = np.sqrt(((got - ref) ** 2).sum(axis=(-1, -2)))
    den = np.sqrt((ref ** 2).sum(axis=(-1, -2)))
    return float((num / np.maximum(den, 1e-30)).max())


def unpack_vc(vc: torch.Tensor, m: int, d: int) -> np.ndarray:
    """Compressed values as the library stores them (blocked records) -> dense float64 [..., m, d]: the
    library's own kvc_unpack_values for device tensors, its kvc_capsule_value_offset for host tensors."""
    from paper_2605_16439_amd import kvcapsule as kv
    if vc.is_cuda:
        dense = kv.kvc_unpack_values(vc, m, d)
        torch.cuda.synchronize()
        return f64(dense)
    flat = f64(vc).reshape(vc.shape[:-2] + (m * d,))
    off = np.array([[kv.lib().kvc_capsule_value_offset(j, c, m, d) for c in range(d)] for j in range(m)])
    return flat[..., off]
