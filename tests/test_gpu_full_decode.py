"""Parity of kvc_attend_full_decode (full-cache "All KV" decode attention, the comparison point of
the paper's efficiency analysis) against the CPU oracle, through the C ABI.

Bar: relative L2 error per output row <= 2e-2 (bf16) / 1e-5 (fp32), every element within 4 x that
of its row's rms, log-sum-exp within 5e-2 / 1e-4; the appended token's k, v land in the cache bit
for bit.
"""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc
from paper_2605_16439_amd import kvcapsule as kv
from paper_2605_16439_amd import synth

from helpers import elem_rel_err, f64, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def make_cache(seed, B, Hkv, cap, d, dtype):
    g = torch.Generator()
    g.manual_seed(synth.BASE_SEED + 31 * seed)
    scale = 0.5 + 3.5 * torch.rand((Hkv, d), generator=g)                  # K channel scales, as in synth
    K = (torch.randn((B, Hkv, cap, d), generator=g) * scale[None, :, None, :]).to(dtype)
    V = torch.randn((B, Hkv, cap, d), generator=g).to(dtype)
    return K.contiguous(), V.contiguous(), scale


def step_inputs(seed, step, B, Hq, Hkv, d, dtype, scale):
    g = torch.Generator()
    g.manual_seed(synth.BASE_SEED + 31 * seed + 7919 * (step + 1))
    q = torch.randn((B, Hq, d), generator=g).to(dtype)
    k = (torch.randn((B, Hkv, d), generator=g) * scale[None]).to(dtype)
    v = torch.randn((B, Hkv, d), generator=g).to(dtype)
    return q, k, v


def run_case(seed, B, Hq, Hkv, d, kv_len, steps=1, dtype=torch.bfloat16, append=True, layout="bhsd",
             scale=0.0, chunk_steps=0, bs=None):
    cap = kv_len + steps
    K, V, chs = make_cache(seed, B, Hkv, cap, d, dtype)
    if layout == "bshd":        # heads interleaved per token, as a backbone's projection output
        gK = K.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
        gV = V.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
        assert not gK.is_contiguous()
    else:
        gK, gV = K.to(DEV), V.to(DEV)
    nbytes = kv.kvc_attend_full_workspace_bytes(B, Hq, Hkv, d, dtype, cap)
    assert nbytes > 0
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=DEV).fill_(0xFF)
    out = torch.zeros((B, Hq, d), dtype=dtype, device=DEV)
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=DEV)
    tol = 1e-5 if dtype == torch.float32 else 2e-2
    bs = list(range(B)) if bs is None else bs
    Kh, Vh = f64(K).copy(), f64(V).copy()
    kv.lib().kvc_dev_full_decode_chunk_steps(chunk_steps)
    t = kv_len
    worst = 0.0
    try:
        for step in range(steps):
            q, kn, vn = step_inputs(seed, step, B, Hq, Hkv, d, dtype, chs)
            if append:
                kv.kvc_attend_full_decode(q.to(DEV), gK, gV, t, kn.to(DEV), vn.to(DEV), scale, out, lse, ws)
                Kh[:, :, t], Vh[:, :, t] = f64(kn), f64(vn)
                t += 1
            else:
                kv.kvc_attend_full_decode(q.to(DEV), gK, gV, t, None, None, scale, out, lse, ws)
            torch.cuda.synchronize()
            ref, lref = orc.attend_full(f64(q)[bs], Kh[bs], Vh[bs], t, scale if scale > 0 else None)
            got, gl = f64(out)[bs], f64(lse)[bs]
            e, ex, el = row_rel_err(got, ref), elem_rel_err(got, ref), float(np.abs(gl - lref).max())
            _say(f"[full] seed {seed} B={B} Hq={Hq} Hkv={Hkv} d={d} t={t} step {step}: row {e:.3e} element {ex:.3e} lse {el:.3e}")
            assert e <= tol and ex <= 4 * tol
            assert el <= (1e-4 if dtype == torch.float32 else 5e-2)
            worst = max(worst, e)
    finally:
        kv.lib().kvc_dev_full_decode_chunk_steps(0)
    # the cache on the device received every appended token, bit for bit, and nothing else changed
    assert np.array_equal(f64(gK), Kh) and np.array_equal(f64(gV), Vh)
    return worst


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (8, 2), (14, 2), (16, 2), (16, 1)])
def test_full_decode_group_sizes(hq, hkv):
    run_case(1 + hq, 2, hq, hkv, 128, 300, steps=2)


@pytest.mark.parametrize("kv_len", [0, 1, 31, 32, 33, 127, 128, 129, 255, 257, 1000])
def test_full_decode_ragged_lengths(kv_len):
    """Lengths around the 32-row wave step and the 128-row workgroup step; kv_len = 0 attends the new
    token alone."""
    run_case(40 + kv_len, 2, 14, 2, 128, kv_len, steps=2)


def test_full_decode_without_append():
    run_case(60, 2, 14, 2, 128, 333, steps=1, append=False)


def test_full_decode_strided_cache_and_explicit_scale():
    run_case(61, 3, 8, 4, 128, 200, steps=2, layout="bshd", scale=0.07)


@pytest.mark.parametrize("chunk_steps", [1, 3, 64])
def test_full_decode_split_sizes(chunk_steps):
    """One step per split (many parts), an odd number of steps per split (the pairwise loop runs one
    masked step), and a single split."""
    run_case(62 + chunk_steps, 2, 14, 2, 128, 1500, steps=1, chunk_steps=chunk_steps)


def test_full_decode_scalar_path_fp32_and_other_head_dim():
    run_case(70, 2, 6, 3, 64, 150, steps=2, dtype=torch.float32)
    run_case(71, 1, 4, 2, 64, 90, steps=1, dtype=torch.bfloat16)


def test_full_decode_long_cache_many_splits():
    """More rows than 64 splits of the default size: the split grows instead."""
    run_case(72, 1, 8, 1, 128, 70000, steps=1)


def test_full_decode_config4_full_size():
    """The headline shape without KVCapsule: B = 4, 28 / 4 heads, 8192 vision + 512 text rows; every
    (batch element, head), first and last decode step of the run (the steps between are run on
    the GPU only)."""
    w = synth.WORKLOADS["qwen2vl"]
    B, Hq, Hkv, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    kv_len = w.n_images * w.n_img_tokens + w.text_len
    run_case(80, B, Hq, Hkv, d, kv_len, steps=1)
    run_case(81, B, Hq, Hkv, d, kv_len + w.steps - 1, steps=1)


def test_full_decode_argument_errors():
    B, Hq, Hkv, d = 1, 4, 2, 128
    K, V, _ = make_cache(90, B, Hkv, 16, d, torch.bfloat16)
    gK, gV = K.to(DEV), V.to(DEV)
    q = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros_like(q)
    ws = torch.empty(kv.kvc_attend_full_workspace_bytes(B, Hq, Hkv, d, torch.bfloat16, 16) + 256,
                     dtype=torch.uint8, device=DEV)
    f = lambda **k: kv.kvc_attend_full_decode(k.get("q", q), gK, gV, k.get("t", 8), k.get("kn"), k.get("vn"), 0.0,
                                              out, None, k.get("ws", ws), check=False)
    kn = torch.zeros((B, Hkv, d), dtype=torch.bfloat16, device=DEV)
    assert f() == kv.KVC_OK
    assert f(t=17) == kv.KVC_ERR_SHAPE
    assert f(t=16, kn=kn, vn=kn) == kv.KVC_ERR_SHAPE          # no room for the new token
    assert f(t=0) == kv.KVC_ERR_SHAPE                          # no key at all
    assert f(kn=kn) == kv.KVC_ERR_NULL
    assert f(ws=torch.empty(512, dtype=torch.uint8, device=DEV)) == kv.KVC_ERR_WORKSPACE
    torch.cuda.synchronize()
