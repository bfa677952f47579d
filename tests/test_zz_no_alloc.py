"""kvc_reconstruct_attend_decode_static (the decode entry point that takes no workspace and allocates
nothing) against kvc_reconstruct_attend_decode on the same inputs, through the C ABI: two calls in
a row, the second on a smaller input, each bit for bit equal to the entry point with a caller-owned
workspace (same kernels, deterministic), and within the usual bar of the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as orc
from paper_2605_16439_amd import kvcapsule as kv
from paper_2605_16439_amd import synth

from helpers import f64, row_rel_err, unpack_vc

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _layer(w, m, packed=False):
    shape = kv.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_img_tokens, w.n_images, m,
                          w.torch_dtype)
    p = synth.make_params(w, m)
    g = {k: v.to(DEV) for k, v in p.items()}
    if packed:      # the packed parameter forms too: the shapes that have a one-pass kernel then take it
        g["theta_packed"], g["U_packed"] = kv.kvc_pack_theta(shape, g["theta"]), kv.kvc_pack_u(shape, g["U"])
    params = kv.make_params(g["key_idx"], g["theta"], g["U"], g["mu"], g.get("theta_packed"), g.get("U_packed"))
    K, V = synth.make_prefill_kv(w)
    Kt, Vt = synth.make_text_cache(w)
    ws = kv.new_workspace(shape, w.text_cap)
    shp = (w.batch, w.n_kv_heads, w.n_images, m, w.head_dim)
    Kc = torch.zeros(shp, dtype=w.torch_dtype, device=DEV)
    Vc = torch.zeros(shp, dtype=w.torch_dtype, device=DEV)
    kv.kvc_compress(shape, params, K.to(DEV), V.to(DEV), 0, Kc, Vc, ws)
    torch.cuda.synchronize()
    return dict(w=w, m=m, shape=shape, p=p, g=g, params=params, Kc=Kc, Vc=Vc, Kt=Kt, Vt=Vt, ws=ws)


def _both(L, step):
    w = L["w"]
    q, kn, vn = (x.to(DEV) for x in synth.make_step_inputs(w, 0, step))
    res = []
    for static in (False, True):
        gKt, gVt = L["Kt"].to(DEV), L["Vt"].to(DEV)
        out = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=w.torch_dtype, device=DEV)
        lse = torch.zeros((w.batch, w.n_q_heads), dtype=torch.float32, device=DEV)
        if static:
            kv.kvc_reconstruct_attend_decode_static(L["shape"], L["params"], q, L["Kc"], L["Vc"], gKt, gVt,
                                                    w.text_len, w.text_cap, kn, vn, 0.0, out, lse)
        else:
            kv.kvc_reconstruct_attend_decode(L["shape"], L["params"], q, L["Kc"], L["Vc"], gKt, gVt,
                                             w.text_len, w.text_cap, kn, vn, 0.0, out, lse, L["ws"])
        torch.cuda.synchronize()
        res.append((f64(out), f64(lse), f64(gKt), f64(gVt)))
    (o0, l0, k0, v0), (o1, l1, k1, v1) = res
    assert np.array_equal(o0, o1) and np.array_equal(l0, l1), "static-scratch call differs from the workspace call"
    assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
    # and both agree with the oracle (common capsule)
    Kt, Vt = f64(L["Kt"]).copy(), f64(L["Vt"]).copy()
    ref, _ = orc.reconstruct_attend_decode(f64(q), f64(L["Kc"]), unpack_vc(L["Vc"], L["m"], w.head_dim),
                                           f64(L["p"]["theta"]), f64(L["p"]["U"]), f64(L["p"]["mu"]),
                                           w.n_img_tokens, Kt, Vt, w.text_len, f64(kn), f64(vn))
    e = row_rel_err(o1, ref)
    print(f"[no-alloc] {w.name}: equal to the workspace call; vs oracle {e:.3e}", flush=True)
    assert e <= (1e-5 if w.dtype == "f32" else 2e-2)


def test_static_scratch_decode_two_calls_second_smaller():
    assert kv.lib().kvc_static_scratch_bytes() == 32 << 20
    big = synth.Workload("noalloc_big", 90, 1, 2, 14, 2, 128, "bf16", 1024, 8, 0.6, 200, 2)
    small = synth.Workload("noalloc_small", 91, 1, 1, 14, 2, 128, "bf16", 256, 2, 0.6, 20, 2)
    A = _layer(big, kv.kvc_compressed_len(1024, 0.6))
    Bs = _layer(small, kv.kvc_compressed_len(256, 0.6))
    _both(A, 0)
    _both(Bs, 0)        # the smaller input right after the larger one: stale scratch must not matter
    _both(A, 1)
    # the one-pass kernel (packed parameter forms) through the same entry point, then the small input again
    taken = kv.lib().kvc_dev_stream_calls()
    _both(_layer(big, kv.kvc_compressed_len(1024, 0.6), packed=True), 0)
    assert kv.lib().kvc_dev_stream_calls() == taken + 2
    _both(Bs, 1)
    # the scalar kernels (fp32) through the same entry point
    tiny = synth.Workload("noalloc_f32", 92, 1, 1, 6, 3, 64, "f32", 40, 3, 0.6, 5, 2)
    _both(_layer(tiny, 16), 0)


def test_static_scratch_refuses_shapes_beyond_its_size():
    w = synth.Workload("noalloc_huge", 93, 1, 64, 28, 4, 128, "bf16", 1024, 64, 0.6, 16, 1)
    shape = kv.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_img_tokens, w.n_images, 410,
                          w.torch_dtype)
    assert kv.kvc_workspace_bytes(shape, w.text_cap) > kv.lib().kvc_static_scratch_bytes()
    x = torch.zeros(4096, dtype=torch.bfloat16, device=DEV)       # never read: the call is refused first
    params = kv.make_params(x, x, x, x)
    st = kv.kvc_reconstruct_attend_decode_static(shape, params, x, x, x, x, x, 1, w.text_cap, None, None, 0.0,
                                                 x, None, check=False)
    assert st == kv.KVC_ERR_WORKSPACE
