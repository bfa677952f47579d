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
    """Compressed values as the library stores them ([..., m*d] records: rows in blocks of 8,
    each block channel-major [d][w]) -> dense float64 [..., m, d].  Index shuffling only."""
    flat = f64(vc).reshape(vc.shape[:-2] + (m * d,)) if vc.dim() >= 2 else f64(vc)
    lead = flat.shape[:-1]
    out = np.empty(lead + (m, d), dtype=np.float64)
    for jb in range((m + 7) // 8):
        w = min(8, m - 8 * jb)
        blk = flat[..., jb * 8 * d: jb * 8 * d + d * w].reshape(lead + (d, w))
        out[..., 8 * jb: 8 * jb + w, :] = np.swapaxes(blk, -1, -2)
    return out
