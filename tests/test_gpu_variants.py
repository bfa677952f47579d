"""Parity of the method's variants against the CPU oracle, through the C ABI: ragged batches
(kvc_reconstruct_attend_decode_ragged), the two-layer key reconstructor (kvc_mlp_hidden + the ordinary
decode step with theta = W2), and the static variant without reconstruction (kvc_static_attend_decode).

Bars as in tests/test_gpu_parity.py: output rows within 1e-5 (fp32) / 2e-2 (bf16) relative L2 error, every
element within 4 x that of its row's rms; the first-layer result within the same relative error per
(b, h, i) block; appended tokens land in the text cache bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc
from paper_2605_16439_amd import kvcapsule as kv
from paper_2605_16439_amd import synth

from helpers import block_rel_err, elem_rel_err, f64, row_rel_err, tol, unpack_vc
from test_gpu_parity import DEV, Layer

pytestmark = pytest.mark.gpu

F32 = synth.Workload("var_f32", 70, 1, 4, 6, 3, 64, "f32", 40, 3, 0.6, 6, 3)
BF16 = synth.Workload("var_bf16", 71, 1, 4, 14, 2, 128, "bf16", 256, 4, 0.6, 50, 3)


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("w,m", [(F32, 16), (BF16, 103)])
def test_ragged_batch(w, m):
    """Sequences with 0 .. I image blocks and text rows from none to the capacity in one call; capsule slots
    and text rows a sequence does not have are filled with NaNs on the device and must not matter."""
    L = Layer(w, m)
    L.compress()
    B, I, cap = w.batch, w.n_images, w.text_cap
    n_images = [I, 0, 1, I - 1][:B]
    text_len = [3, w.text_len, 0, cap - 1][:B]
    gKc, gVc = L.gKc.clone(), L.gVc.clone()
    Kc_h, Vc_h = f64(gKc), unpack_vc(gVc, m, w.head_dim)
    for b in range(B):                      # poison what the sequence does not own
        gKc[b, :, n_images[b]:] = float("nan")
        gVc[b, :, n_images[b]:] = float("nan")
        L.gKt[b, :, text_len[b]:] = float("nan")
        L.gVt[b, :, text_len[b]:] = float("nan")
    ni = torch.tensor(n_images, dtype=torch.int32, device=DEV)
    tl = torch.tensor(text_len, dtype=torch.int32, device=DEV)
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    th, U, mu = f64(L.p["theta"]), f64(L.p["U"]), f64(L.p["mu"])
    for step in range(1):
        q, kn, vn = synth.make_step_inputs(w, 0, step)
        kv.kvc_reconstruct_attend_decode_ragged(L.shape, L.params, q.to(DEV), gKc, gVc, L.gKt, L.gVt, ni, tl, cap,
                                                kn.to(DEV), vn.to(DEV), 0.0, L.out, L.lse, L.ws)
        torch.cuda.synchronize()
        ref, lref = orc.reconstruct_attend_decode_ragged(f64(q), Kc_h, Vc_h, th, U, mu, w.n_img_tokens, n_images,
                                                         text_len, Kt, Vt, f64(kn), f64(vn))
        out, lse = f64(L.out), f64(L.lse)
        e, ex = row_rel_err(out, ref), elem_rel_err(out, ref)
        _say(f"[ragged] {w.name}: row {e:.3e} element {ex:.3e} lse {np.abs(lse - lref).max():.3e}")
        assert np.all(np.isfinite(out))
        assert e <= tol(w) and ex <= 4 * tol(w)
        assert np.abs(lse - lref).max() <= (1e-4 if w.dtype == "f32" else 5e-2)
        for b in range(B):                  # the new token went to the sequence's own row
            assert np.array_equal(f64(L.gKt)[b, :, text_len[b]], f64(kn)[b])
            assert np.array_equal(f64(L.gVt)[b, :, text_len[b]], f64(vn)[b])
    # a uniform batch through the ragged entry point equals the uniform entry point bit for bit (both take
    # the matrix-core kernels where the shape has them, the scalar ones elsewhere)
    L2 = Layer(w, m)
    L2.compress()
    q, kn, vn = synth.make_step_inputs(w, 0, 1)
    a, la = L2.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    L3 = Layer(w, m)
    L3.compress()
    kv.kvc_reconstruct_attend_decode_ragged(L3.shape, L3.params, q.to(DEV), L3.gKc, L3.gVc, L3.gKt, L3.gVt,
                                            torch.full((B,), I, dtype=torch.int32, device=DEV),
                                            torch.full((B,), w.text_len, dtype=torch.int32, device=DEV), cap,
                                            kn.to(DEV), vn.to(DEV), 0.0, L3.out, L3.lse, L3.ws)
    torch.cuda.synchronize()
    assert np.array_equal(f64(L3.out), a) and np.array_equal(f64(L3.lse), la)


RAG_HEAD = synth.Workload("rag_headline", 72, 1, 4, 7, 1, 128, "bf16", 1024, 8, 0.6, 300, 2)     # G = 7, merged part records
RAG_G1 = synth.Workload("rag_g1", 73, 1, 12, 2, 2, 128, "bf16", 576, 5, 0.6, 140, 2)              # G = 1: 32 image blocks per workgroup
RAG_VIDEO = synth.Workload("rag_video", 74, 1, 2, 14, 2, 128, "bf16", 256, 24, 0.6, 260, 2)       # four row tiles per workgroup


@pytest.mark.parametrize("w,m,n_images,text_len,append", [
    (RAG_HEAD, 410, [8, 0, 1, 3], [300, 0, 129, 17], True),
    (RAG_HEAD, 410, [8, 0, 1, 3], [302, 1, 128, 17], False),
    (RAG_G1, 231, [5, 0, 1, 3, 5, 2, 0, 4, 1, 5, 3, 0], [140, 0, 1, 127, 128, 129, 7, 64, 141, 33, 90, 2], True),
    (RAG_VIDEO, 103, [24, 5], [260, 3], True),
    (RAG_VIDEO, 103, [0, 0], [0, 200], True),
])
def test_ragged_batch_on_the_matrix_core_kernels(w, m, n_images, text_len, append):
    """Shapes that take the matrix-core kernels (fused and separate first launches, merged and per-block part
    records, 2 to 64 image blocks per workgroup): blocks and text rows a sequence does not have hold NaNs."""
    L = Layer(w, m)
    L.compress()
    B, I, cap = w.batch, w.n_images, w.text_cap
    gKc, gVc = L.gKc.clone(), L.gVc.clone()
    Kc_h, Vc_h = f64(gKc), unpack_vc(gVc, m, w.head_dim)
    rows = [t + (1 if append else 0) for t in text_len]
    for b in range(B):
        gKc[b, :, n_images[b]:] = float("nan")
        gVc[b, :, n_images[b]:] = float("nan")
        L.gKt[b, :, rows[b]:] = float("nan")
        L.gVt[b, :, rows[b]:] = float("nan")
    ni = torch.tensor(n_images, dtype=torch.int32, device=DEV)
    tl = torch.tensor(text_len, dtype=torch.int32, device=DEV)
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    th, U, mu = f64(L.p["theta"]), f64(L.p["U"]), f64(L.p["mu"])
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    gkn, gvn = (kn.to(DEV), vn.to(DEV)) if append else (None, None)
    # twice: the first call on a fresh workspace may find garbage in the arrival counters and compute without
    # waiting (correct, counted); the second must not (appending the same token again changes nothing)
    for rep in range(2):
        alone = kv.lib().kvc_dev_decode_fallbacks()
        kv.kvc_reconstruct_attend_decode_ragged(L.shape, L.params, q.to(DEV), gKc, gVc, L.gKt, L.gVt, ni, tl, cap,
                                                gkn, gvn, 0.0, L.out, L.lse, L.ws)
        torch.cuda.synchronize()
    ref, lref = orc.reconstruct_attend_decode_ragged(f64(q), Kc_h, Vc_h, th, U, mu, w.n_img_tokens, n_images,
                                                     text_len, Kt, Vt, f64(kn) if append else None,
                                                     f64(vn) if append else None)
    out, lse = f64(L.out), f64(L.lse)
    e, ex = row_rel_err(out, ref), elem_rel_err(out, ref)
    _say(f"[ragged, matrix cores] {w.name} append={append}: row {e:.3e} element {ex:.3e} lse {np.abs(lse - lref).max():.3e}")
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
    assert e <= tol(w) and ex <= 4 * tol(w)
    assert np.abs(lse - lref).max() <= 5e-2
    if append:
        for b in range(B):
            assert np.array_equal(f64(L.gKt)[b, :, text_len[b]], f64(kn)[b])
            assert np.array_equal(f64(L.gVt)[b, :, text_len[b]], f64(vn)[b])
    assert kv.lib().kvc_dev_decode_fallbacks() == alone


def test_ragged_argument_errors():
    w = F32
    L = Layer(w, 16)
    x = torch.zeros(w.batch, dtype=torch.int32, device=DEV)
    q, kn, vn = (t.to(DEV) for t in synth.make_step_inputs(w, 0, 0))
    f = lambda ni=x, tl=x, cap=w.text_cap: kv.kvc_reconstruct_attend_decode_ragged(
        L.shape, L.params, q, L.gKc, L.gVc, L.gKt, L.gVt, ni, tl, cap, kn, vn, 0.0, L.out, L.lse, L.ws, check=False)
    assert f(cap=0) == kv.KVC_ERR_SHAPE
    st = kv.lib().kvc_reconstruct_attend_decode_ragged(None, None, None, None, None, None, None, None, None, 4, None,
                                                       None, 0.0, None, None, None, 0, None)
    assert st == kv.KVC_ERR_NULL


@pytest.mark.parametrize("w,m,act", [(F32, 16, kv.KVC_ACT_GELU), (F32, 16, kv.KVC_ACT_RELU),
                                     (BF16, 103, kv.KVC_ACT_GELU), (BF16, 103, kv.KVC_ACT_IDENTITY)])
def test_two_layer_key_reconstructor(w, m, act):
    """compress -> first layer (kvc_mlp_hidden) -> decode with theta = W2, against the oracle's first layer
    and its definitional reconstruct + attend on the stored hidden rows."""
    L = Layer(w, m)
    L.compress()
    g = torch.Generator()
    g.manual_seed(synth.BASE_SEED + 4242 + m)
    W1 = (torch.randn((w.n_kv_heads, m, m), generator=g) * (1.0 / m) ** 0.5).to(w.torch_dtype)
    gW1 = W1.to(DEV)
    H = torch.zeros_like(L.gKc)
    kv.kvc_mlp_hidden(L.shape, gW1, act, L.gKc, H)
    torch.cuda.synchronize()
    code = orc.STORE_F32 if w.dtype == "f32" else orc.STORE_BF16
    H_ref = orc.mlp_hidden(f64(L.gKc), f64(W1), act, code)
    e = block_rel_err(f64(H), H_ref)
    _say(f"[mlp] {w.name} act={act}: first layer block rel err {e:.3e}")
    assert e <= tol(w)
    # decode on the common stored rows: W2 is the layer's theta
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    kv.kvc_reconstruct_attend_decode(L.shape, L.params, q.to(DEV), H, L.gVc, L.gKt, L.gVt, w.text_len, w.text_cap,
                                     kn.to(DEV), vn.to(DEV), 0.0, L.out, L.lse, L.ws)
    torch.cuda.synchronize()
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    ref, _ = orc.reconstruct_attend_decode(f64(q), f64(H), unpack_vc(L.gVc, m, w.head_dim), f64(L.p["theta"]),
                                           f64(L.p["U"]), f64(L.p["mu"]), w.n_img_tokens, Kt, Vt, w.text_len,
                                           f64(kn), f64(vn))
    out = f64(L.out)
    e2, ex = row_rel_err(out, ref), elem_rel_err(out, ref)
    _say(f"[mlp] {w.name} act={act}: decode row {e2:.3e} element {ex:.3e}")
    assert e2 <= tol(w) and ex <= 4 * tol(w)
    assert kv.kvc_mlp_hidden(L.shape, gW1, 7, L.gKc, H, check=False) == kv.KVC_ERR_SHAPE
    assert kv.kvc_mlp_hidden(L.shape, gW1, act, L.gKc, L.gKc, check=False) == kv.KVC_ERR_SHAPE


@pytest.mark.parametrize("w,m", [(F32, 16), (BF16, 103)])
def test_static_variant_without_reconstruction(w, m):
    L = Layer(w, m)
    L.compress()
    Kc_h, Vc_h = f64(L.gKc), unpack_vc(L.gVc, m, w.head_dim)
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    t = w.text_len
    for step in range(2):
        q, kn, vn = synth.make_step_inputs(w, 0, step)
        kv.kvc_static_attend_decode(L.shape, q.to(DEV), L.gKc, L.gVc, L.gKt, L.gVt, t, w.text_cap, kn.to(DEV),
                                    vn.to(DEV), 0.0, L.out, L.lse, L.ws)
        torch.cuda.synchronize()
        ref, lref = orc.static_attend_decode(f64(q), Kc_h, Vc_h, Kt, Vt, t, f64(kn), f64(vn))
        t += 1
        out, lse = f64(L.out), f64(L.lse)
        e, ex = row_rel_err(out, ref), elem_rel_err(out, ref)
        _say(f"[static] {w.name} step {step}: row {e:.3e} element {ex:.3e} lse {np.abs(lse - lref).max():.3e}")
        assert e <= tol(w) and ex <= 4 * tol(w)
        assert np.abs(lse - lref).max() <= (1e-4 if w.dtype == "f32" else 5e-2)
    assert np.array_equal(f64(L.gKt)[:, :, :t], Kt[:, :, :t]) and np.array_equal(f64(L.gVt)[:, :, :t], Vt[:, :, :t])
