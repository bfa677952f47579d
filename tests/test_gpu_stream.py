"""Parity of the one-pass ("stream") decode kernel against the CPU oracle, through the C ABI: the call is
kvc_reconstruct_attend_decode with kvc_params.theta_packed set (kvc_pack_theta), forced onto the one-pass
kernel with kvc_dev_stream_decode(1) so that small test shapes take it too.

Bars as in tests/test_gpu_parity.py (bf16): output rows within 2e-2 relative L2 error, every element within
4 x that of its row's rms, lse within 5e-2; appended tokens land in the text cache bit for bit; theta packed
by the library equals the layout function kvc_capsule_value_offset(j, pos, m, n) bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc
from paper_2605_16439_amd import kvcapsule as kv
from paper_2605_16439_amd import synth

from helpers import elem_rel_err, f64, row_rel_err, tol, unpack_vc
from test_gpu_parity import DEV, Layer

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def _force_stream():
    kv.lib().kvc_dev_stream_decode(1)
    yield
    kv.lib().kvc_dev_stream_decode(-1)


def _wl(name, idx, batch, hkv, n_images, text_len, steps=2):
    return synth.Workload(name, idx, 1, batch, 7 * hkv, hkv, 128, "bf16", 1024, n_images, 0.6, text_len, steps)


def _packed_layer(w, m):
    L = Layer(w, m)
    L.theta_packed = kv.kvc_pack_theta(L.shape, L.g["theta"])
    L.U_packed = kv.kvc_pack_u(L.shape, L.g["U"])
    L.params = kv.make_params(L.g["key_idx"], L.g["theta"], L.g["U"], L.g["mu"], L.theta_packed, L.U_packed)
    L.compress()
    return L


def _run(L, w, m, steps, append=True, t0=None, lse_tol=5e-2):
    th, U, mu = f64(L.p["theta"]), f64(L.p["U"]), f64(L.p["mu"])
    Kc_h, Vc_h = f64(L.gKc), unpack_vc(L.gVc, m, w.head_dim)
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    t = w.text_len if t0 is None else t0
    taken = kv.lib().kvc_dev_stream_calls()
    for step in range(steps):
        q, kn, vn = synth.make_step_inputs(w, 0, step)
        if append:
            out, lse = L.decode(q.to(DEV), t, kn.to(DEV), vn.to(DEV))
            ref, lref = orc.reconstruct_attend_decode(f64(q), Kc_h, Vc_h, th, U, mu, w.n_img_tokens, Kt, Vt, t,
                                                      f64(kn), f64(vn))
        else:
            out, lse = L.decode(q.to(DEV), t)
            ref, lref = orc.reconstruct_attend_decode(f64(q), Kc_h, Vc_h, th, U, mu, w.n_img_tokens,
                                                      Kt if t else None, Vt if t else None, t)
        e, ex, el = row_rel_err(out, ref), elem_rel_err(out, ref), np.abs(lse - lref).max()
        _say(f"[stream] {w.name} m={m} t={t} append={append} step {step}: row {e:.3e} element {ex:.3e} lse {el:.3e}")
        assert np.all(np.isfinite(out))
        assert e <= tol(w) and ex <= 4 * tol(w) and el <= lse_tol
        if append:
            assert np.array_equal(f64(L.gKt)[:, :, t], f64(kn)) and np.array_equal(f64(L.gVt)[:, :, t], f64(vn))
            t += 1
    assert kv.lib().kvc_dev_stream_calls() == taken + steps, "the one-pass kernel must have served these calls"


def test_pack_theta_layout():
    w = _wl("st_pack", 80, 1, 2, 2, 8)
    for m in (410, 205, 7, 8):
        L = Layer(w, m)
        packed = kv.kvc_pack_theta(L.shape, L.g["theta"])
        torch.cuda.synchronize()
        n = w.n_img_tokens
        off = np.array([[kv.lib().kvc_capsule_value_offset(j, p, m, n) for p in range(0, n, 37)] for j in range(m)])
        src = L.p["theta"].view(torch.int16).numpy().reshape(w.n_kv_heads, m * n)
        got = packed.cpu().view(torch.int16).numpy().reshape(w.n_kv_heads, m * n)
        for h in range(w.n_kv_heads):
            dense = src[h].reshape(m, n)[:, ::37]
            assert np.array_equal(got[h][off], dense)
        # U: the same layout with the roles of rows and positions exchanged
        packed_u = kv.kvc_pack_u(L.shape, L.g["U"])
        torch.cuda.synchronize()
        off_u = np.array([[kv.lib().kvc_capsule_value_offset(p, j, n, m) for p in range(0, n, 37)] for j in range(m)])
        src_u = L.p["U"].view(torch.int16).numpy().reshape(w.n_kv_heads, m * n)
        got_u = packed_u.cpu().view(torch.int16).numpy().reshape(w.n_kv_heads, m * n)
        for h in range(w.n_kv_heads):
            assert np.array_equal(got_u[h][off_u], src_u[h].reshape(m, n)[:, ::37])


# compressed lengths over the compiled instances (1 .. 21 steps of 32 rows): a short last block of every width
# class, no short block, a last 16-row tile that is missing, the shortest and longest length of an instance
@pytest.mark.parametrize("m", [410, 416, 400, 385, 415, 393, 205, 193, 224, 615, 609, 640, 1, 7, 31, 33, 100, 300, 672, 673, 1000, 1024])
def test_compressed_lengths(m):
    w = _wl("st_len", 81, 2, 2, 4, 77)
    L = _packed_layer(w, m)
    # a single compressed row: every logit of a block is one bf16-rounded score times a row of theta with entries
    # of order one, so the logits (and lse) carry the score's rounding, 2^-9 of logits of +-30
    _run(L, w, m, 2, lse_tol=5e-2 if m > 1 else 2e-1)


@pytest.mark.parametrize("text_len,append", [(0, True), (0, False), (1, True), (15, False), (16, True), (300, True),
                                             (1000, True)])
def test_text_lengths(text_len, append):
    w = _wl("st_text", 82, 1, 2, 8 if text_len > 500 else 2, text_len, 3)
    L = _packed_layer(w, 410)
    _run(L, w, 410, 3 if append else 1, append)


def test_headline_shape_every_element():
    w = synth.WORKLOADS["qwen2vl"].with_(layers=1, steps=2)
    L = _packed_layer(w, 410)
    th, U, mu = f64(L.p["theta"]), f64(L.p["U"]), f64(L.p["mu"])
    Kt, Vt = f64(L.Kt).copy(), f64(L.Vt).copy()
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    out, lse = L.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    # the same call on the four-kernel form (no packed theta): both within the bar of the oracle, and close
    L2 = Layer(w, 410)
    L2.compress()
    out2, lse2 = L2.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    bs, hs = [0, w.batch - 1], [0, w.n_kv_heads - 1]
    G = w.n_q_heads // w.n_kv_heads
    gs = [h * G + g for h in hs for g in range(G)]
    sel, selq = np.ix_(bs, hs), np.ix_(bs, gs)
    ref, lref = orc.reconstruct_attend_decode(f64(q)[selq], f64(L.gKc)[sel], unpack_vc(L.gVc, 410, 128)[sel], th[hs], U[hs],
                                              mu[hs], w.n_img_tokens, Kt[sel].copy(), Vt[sel].copy(), w.text_len,
                                              f64(kn)[sel], f64(vn)[sel])
    e, ex = row_rel_err(out[selq], ref), elem_rel_err(out[selq], ref)
    e2 = row_rel_err(out2[selq], ref)
    _say(f"[stream] headline: row {e:.3e} element {ex:.3e} lse {np.abs(lse[selq] - lref).max():.3e}; four-kernel form row {e2:.3e}")
    assert e <= tol(w) and ex <= 4 * tol(w) and np.abs(lse[selq] - lref).max() <= 5e-2
    assert row_rel_err(out, out2) <= 2 * tol(w)


@pytest.mark.parametrize("w,m", [(synth.Workload("st_other", 83, 1, 2, 14, 2, 128, "bf16", 256, 4, 0.6, 50, 2), 103),
                                 (synth.Workload("st_576", 84, 1, 2, 14, 2, 128, "bf16", 576, 2, 0.6, 20, 2), 231),
                                 (synth.Workload("st_g1", 85, 1, 3, 8, 8, 128, "bf16", 576, 5, 0.6, 150, 2), 229),
                                 (synth.Workload("st_vid", 86, 1, 2, 14, 2, 128, "bf16", 256, 24, 0.6, 260, 2), 103)])
def test_shapes_without_an_instance_take_the_other_kernels(w, m):
    """The packed forms are optional help: a shape the one-pass kernel is not compiled for (other block sizes and
    group sizes) runs the four-kernel form, which reads U in the packed form where it is given (same operands in
    the same order) and gives the same result as the call without them, bit for bit."""
    L = _packed_layer(w, m)
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    a, la = L.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    L2 = Layer(w, m)
    L2.compress()
    b, lb = L2.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_workgroups_that_do_not_wait_compute_every_share_themselves():
    """The hand-over of the scores between the workgroups of a group is bounded: with the wait set to zero every
    workgroup computes all shares alone (counted), same result; with the normal wait nobody does."""
    w = _wl("st_alone", 85, 2, 2, 4, 60)
    L = _packed_layer(w, 410)
    L.ws.zero_()                                         # (a fresh allocation may hold anything: one slow call)
    before = kv.lib().kvc_dev_decode_fallbacks()
    _run(L, w, 410, 2)
    assert kv.lib().kvc_dev_decode_fallbacks() == before, "normal calls must not fall back"
    kv.lib().kvc_dev_decode_knobs(-1, -1, 0)
    try:
        L2 = _packed_layer(w, 410)
        _run(L2, w, 410, 2)
        assert kv.lib().kvc_dev_decode_fallbacks() > before
    finally:
        kv.lib().kvc_dev_decode_knobs(-1, -1, 2000)


def test_replayed_from_a_hip_graph_with_garbage_in_the_workspace():
    """The call only enqueues kernels, so it can be captured; replays with the workspace (arrival counters
    included) overwritten in between must reproduce the eager result: a counter word that holds something else
    ends in the compute-alone path, and the call's last kernel leaves zeros behind."""
    w = _wl("st_graph", 86, 1, 2, 4, 40)
    L = _packed_layer(w, 205)
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    gq, gkn, gvn = q.to(DEV), kn.to(DEV), vn.to(DEV)
    taken = kv.lib().kvc_dev_stream_calls()
    eager, _ = L.decode(gq, w.text_len, gkn, gvn)
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            kv.kvc_reconstruct_attend_decode(L.shape, L.params, gq, L.gKc, L.gVc, L.gKt, L.gVt, w.text_len, w.text_cap,
                                             gkn, gvn, 0.0, L.out, L.lse, L.ws, stream=s)
    torch.cuda.synchronize()
    assert kv.lib().kvc_dev_stream_calls() == taken + 2
    for rep in range(3):
        L.out.zero_()
        L.ws.fill_(0x5A if rep != 1 else 0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(f64(L.out), eager), f"replay {rep} differs from the eager call"
        g.replay()                                         # and again on the zeros the first replay left
        torch.cuda.synchronize()
        assert np.array_equal(f64(L.out), eager), f"second replay {rep} differs from the eager call"


@pytest.mark.parametrize("n_images,text_len,append", [
    ([8, 0, 1, 3], [300, 0, 129, 17], True),
    ([8, 0, 1, 3], [302, 1, 128, 17], False),
    ([0, 0, 5, 8], [0, 200, 301, 64], True),
])
def test_ragged_batch(n_images, text_len, append):
    """kvc_reconstruct_attend_decode_ragged on the one-pass kernel: sequences with their own numbers of image
    blocks (odd counts split a workgroup's pair) and text rows; capsule slots and text rows a sequence does not
    have hold NaNs on the device and must not matter."""
    w = synth.Workload("st_rag", 87, 1, 4, 14, 2, 128, "bf16", 1024, 8, 0.6, 302, 2)
    m = 410
    L = _packed_layer(w, m)
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
    taken = kv.lib().kvc_dev_stream_calls()
    for rep in range(2):        # appending the same token again changes nothing
        kv.kvc_reconstruct_attend_decode_ragged(L.shape, L.params, q.to(DEV), gKc, gVc, L.gKt, L.gVt, ni, tl, cap,
                                                gkn, gvn, 0.0, L.out, L.lse, L.ws)
        torch.cuda.synchronize()
    assert kv.lib().kvc_dev_stream_calls() == taken + 2
    ref, lref = orc.reconstruct_attend_decode_ragged(f64(q), Kc_h, Vc_h, th, U, mu, w.n_img_tokens, n_images,
                                                     text_len, Kt, Vt, f64(kn) if append else None,
                                                     f64(vn) if append else None)
    out, lse = f64(L.out), f64(L.lse)
    e, ex = row_rel_err(out, ref), elem_rel_err(out, ref)
    _say(f"[stream, ragged] append={append}: row {e:.3e} element {ex:.3e} lse {np.abs(lse - lref).max():.3e}")
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
    assert e <= tol(w) and ex <= 4 * tol(w) and np.abs(lse - lref).max() <= 5e-2
    if append:
        for b in range(B):
            assert np.array_equal(f64(L.gKt)[b, :, text_len[b]], f64(kn)[b])
            assert np.array_equal(f64(L.gVt)[b, :, text_len[b]], f64(vn)[b])


def test_ragged_uniform_batch_equals_the_uniform_call():
    w = _wl("st_ragu", 88, 2, 2, 4, 90)
    L = _packed_layer(w, 410)
    q, kn, vn = synth.make_step_inputs(w, 0, 0)
    a, la = L.decode(q.to(DEV), w.text_len, kn.to(DEV), vn.to(DEV))
    L2 = _packed_layer(w, 410)
    kv.kvc_reconstruct_attend_decode_ragged(L2.shape, L2.params, q.to(DEV), L2.gKc, L2.gVc, L2.gKt, L2.gVt,
                                            torch.full((w.batch,), w.n_images, dtype=torch.int32, device=DEV),
                                            torch.full((w.batch,), w.text_len, dtype=torch.int32, device=DEV),
                                            w.text_cap, kn.to(DEV), vn.to(DEV), 0.0, L2.out, L2.lse, L2.ws)
    torch.cuda.synchronize()
    assert np.array_equal(f64(L2.out), a) and np.array_equal(f64(L2.lse), la)


def test_more_workgroups_than_compute_units():
    """512 workgroups (two rounds over the chip): the four workgroups of a group are dealt out next to each other,
    so they still meet; no fall-back after the first call."""
    w = _wl("st_big", 89, 16, 2, 8, 70)
    L = _packed_layer(w, 205)
    L.ws.zero_()
    before = kv.lib().kvc_dev_decode_fallbacks()
    _run(L, w, 205, 2)
    assert kv.lib().kvc_dev_decode_fallbacks() == before


@pytest.mark.parametrize("g,m", [(4, 410), (6, 410), (8, 410), (4, 77), (6, 205), (8, 615)])
def test_other_group_sizes(g, m):
    """The kernel is compiled for 4, 6, 7 and 8 query heads per KV head (four image blocks per workgroup for 4,
    two otherwise)."""
    w = synth.Workload("st_g%d" % g, 90 + g, 1, 2, g * 2, 2, 128, "bf16", 1024, 4, 0.6, 70, 2)
    L = _packed_layer(w, m)
    _run(L, w, m, 2)
