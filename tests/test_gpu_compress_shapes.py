"""Parity of the matrix-core compress kernel against the CPU oracle over its launch shapes, through the C ABI:
4 and 8 wavefronts per workgroup, one to several workgroups per image block, block lengths of one to five
64-position tiles (the loop's prefetching steps and each of its three tails), compressed lengths around the
16-row tile and the 8-row output block.

Bar: retained keys bit for bit; compressed values within 2e-2 relative error per (b, h, i) block (bf16
storage, fp32 accumulation, one rounding) and every element within 4 x that of its block's rms.
"""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc
from paper_2605_16439_amd import kvcapsule as kv
from paper_2605_16439_amd import synth

from helpers import block_rel_err, f64, store_code, tol, unpack_vc
from test_gpu_parity import Layer

pytestmark = pytest.mark.gpu


@pytest.fixture
def knobs():
    yield kv.lib().kvc_dev_compress_knobs
    kv.lib().kvc_dev_compress_knobs(0, 0)


def run_case(w, m, waves, jt, knobs, pre=0, post=0):
    print(f"[compress] {w.name} n={w.n_img_tokens} I={w.n_images} m={m} waves={waves} jt={jt}", flush=True)
    knobs(waves, jt)
    L = Layer(w, m, pre=pre, post=post)
    L.gKc.fill_(float("nan"))
    L.gVc.fill_(float("nan"))
    L.compress()
    Kc_ref, Vc_ref = orc.compress(f64(L.K), f64(L.V), L.p["key_idx"].numpy(), f64(L.p["U"]), f64(L.p["mu"]),
                                  w.n_img_tokens, w.n_images, pre, store_code(w))
    gKc, gVc = f64(L.gKc), unpack_vc(L.gVc, m, w.head_dim)
    assert np.array_equal(gKc, Kc_ref)
    e = block_rel_err(gVc, Vc_ref)
    rms = np.sqrt((Vc_ref ** 2).mean(axis=(-1, -2), keepdims=True))
    ex = float((np.abs(gVc - Vc_ref) / np.maximum(rms, 1e-30)).max())
    print(f"[compress]   block rel err {e:.3e} worst element / block rms {ex:.3e}", flush=True)
    assert e <= tol(w) and ex <= 4 * tol(w)


def wl(n, I, B=1, hkv=2):
    return synth.Workload(f"cs_n{n}", 90, 1, B, 2 * hkv, hkv, 128, "bf16", n, I, 0.6, 4, 1)


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("n", [64, 128, 192, 256, 320])
def test_block_lengths_cover_every_loop_tail(n, waves, knobs):
    run_case(wl(n, 3), min(n, 103), waves, 0, knobs)


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("m", [1, 7, 8, 15, 16, 17, 63, 64, 65, 127, 130, 255, 256])
def test_compressed_lengths_around_tile_and_block_edges(m, waves, knobs):
    run_case(wl(256, 2), m, waves, 0, knobs)


@pytest.mark.parametrize("waves,jt", [(4, 1), (4, 2), (4, 3), (4, 7), (8, 1), (8, 2), (8, 3), (8, 5), (8, 26)])
def test_workgroups_per_image_block(waves, jt, knobs):
    """m = 410 (26 tiles of 16 rows): every share of tiles per workgroup, also one that leaves the last
    workgroups of a block without rows (26 workgroups of one tile: the kernel's minimum is two here)."""
    run_case(wl(1024, 2), 410, waves, jt, knobs)


@pytest.mark.parametrize("waves", [4, 8])
def test_workgroup_count_not_a_multiple_of_eight_and_offset_span(waves, knobs):
    """3 image blocks x 1 x 1 heads: the XCD-contiguous numbering is off; vision span inside a longer
    prefill sequence."""
    w = synth.Workload("cs_odd", 91, 1, 1, 2, 1, 128, "bf16", 128, 3, 0.6, 4, 1)
    run_case(w, 77, waves, 0, knobs, pre=5, post=9)


def test_headline_shape_both_forms(knobs):
    w = synth.WORKLOADS["qwen2vl"]
    for waves in (4, 8):
        knobs(waves, 0)
        L = Layer(w, 410)
        L.compress()
        bs, hs = [0, w.batch - 1], [1, w.n_kv_heads - 1]
        sel = np.ix_(bs, hs)
        Kc_ref, Vc_ref = orc.compress(f64(L.K)[sel], f64(L.V)[sel], L.p["key_idx"].numpy(), f64(L.p["U"])[hs],
                                      f64(L.p["mu"])[hs], w.n_img_tokens, w.n_images, 0, store_code(w))
        assert np.array_equal(f64(L.gKc)[sel], Kc_ref)
        e = block_rel_err(unpack_vc(L.gVc, 410, w.head_dim)[sel], Vc_ref)
        print(f"[compress] qwen2vl waves={waves}: block rel err {e:.3e}", flush=True)
        assert e <= tol(w)
