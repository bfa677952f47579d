#!/usr/bin/env python3
"""Benchmark of the KVCapsule decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen2vl] [--compression 0.6]

A step is one new token for the whole batch through ALL layers of the workload: per layer
one kvc_reconstruct_attend_decode call (text cache growing by one token per step), after a
one-off kvc_compress pass per layer that builds the capsules (timed separately and reported
in "compress").  Every layer has its own capsule, text cache and parameters, so a step
sweeps the whole working set and no layer is cache-resident when it is revisited.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E peak


def algorithmic_bytes(w, m, t_avg, b=2):
    """HBM bytes one layer-step must move: capsule + text cache + parameters + q/out."""
    capsule = 2 * w.batch * w.n_kv_heads * w.n_images * m * w.head_dim * b
    text = 2 * w.batch * w.n_kv_heads * t_avg * w.head_dim * b
    params = w.n_kv_heads * (2 * m * w.n_img_tokens + w.head_dim) * b
    qout = 2 * w.batch * w.n_q_heads * w.head_dim * b
    return capsule + text + params + qout


def read_traffic():
    """Measured HBM bytes per decode call from the committed rocprofv3 counter summary."""
    path = os.path.join(ROOT, "profiles", "decode_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="qwen2vl")
    ap.add_argument("--compression", type=float, default=0.6)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--generic", action="store_true", help="force the scalar kernels")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="also run 3 plain device copies of this many MiB (counter calibration "
                         "for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "--gpus %d is not supported -- run with --gpus 1" % args.gpus)

    import torch

    from paper_2605_16439_amd import kvcapsule as kv
    from paper_2605_16439_amd import synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload].with_(compression=args.compression)
    if args.layers:
        w = w.with_(layers=args.layers)
    K, W = args.steps, args.warmup
    m = kv.kvc_compressed_len(w.n_img_tokens, w.compression)
    L = w.layers
    cap = w.text_len + K
    shape = kv.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_img_tokens,
                          w.n_images, m, w.torch_dtype)
    ws = kv.new_workspace(shape, cap, dev)
    dt = w.torch_dtype

    # ---- build the per-layer state on the device: parameters, capsule, text cache ------------
    layers = []
    cshape = (w.batch, w.n_kv_heads, w.n_images, m, w.head_dim)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    comp_ms = 0.0
    for l in range(L):
        p = synth.make_params(w, m, l, device=dev)
        params = kv.make_params(p["key_idx"], p["theta"], p["U"], p["mu"])
        Kp, Vp = synth.make_prefill_kv(w, l, 0, 0, device=dev)
        Kc = torch.empty(cshape, dtype=dt, device=dev)
        Vc = torch.empty(cshape, dtype=dt, device=dev)
        e0, e1 = ev(), ev()
        if l == 0:      # untimed first call (module load)
            kv.kvc_compress(shape, params, Kp, Vp, 0, Kc, Vc, ws, generic=args.generic)
        e0.record()
        kv.kvc_compress(shape, params, Kp, Vp, 0, Kc, Vc, ws, generic=args.generic)
        e1.record()
        e1.synchronize()
        comp_ms += e0.elapsed_time(e1)
        Kt, Vt = synth.make_text_cache(w, l, device=dev, cap=cap)
        layers.append(dict(p=p, params=params, Kc=Kc, Vc=Vc, Kt=Kt, Vt=Vt))
        del Kp, Vp
    g = torch.Generator(device=dev)
    g.manual_seed(synth.BASE_SEED + 999)
    q_all = torch.randn((W + K, L, w.batch, w.n_q_heads, w.head_dim), generator=g, device=dev).to(dt)
    kn_all = torch.randn((W + K, L, w.batch, w.n_kv_heads, w.head_dim), generator=g, device=dev).to(dt)
    vn_all = torch.randn((W + K, L, w.batch, w.n_kv_heads, w.head_dim), generator=g, device=dev).to(dt)
    out = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=dt, device=dev)

    # argument tuples are marshalled once, so the timed loop is one foreign call per layer
    import ctypes
    fn = kv.lib().kvc_reconstruct_attend_decode_generic if args.generic else \
        kv.lib().kvc_reconstruct_attend_decode
    wp, wb = kv._ws(ws)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    shp_ref = ctypes.byref(shape)
    vp = ctypes.c_void_p

    def marshal(s, l, t):
        Lr = layers[l]
        return (shp_ref, ctypes.byref(Lr["params"]), vp(q_all[s, l].data_ptr()),
                vp(Lr["Kc"].data_ptr()), vp(Lr["Vc"].data_ptr()), vp(Lr["Kt"].data_ptr()),
                vp(Lr["Vt"].data_ptr()), t, cap, vp(kn_all[s, l].data_ptr()),
                vp(vn_all[s, l].data_ptr()), ctypes.c_float(0.0), vp(out[l].data_ptr()), None,
                wp, wb, stream)

    warm = [[marshal(s, l, w.text_len) for l in range(L)] for s in range(W)]
    timed = [[marshal(W + s, l, w.text_len + s) for l in range(L)] for s in range(K)]

    def layer_step(a):
        st = fn(*a)
        if st != kv.KVC_OK:
            raise kv.KvcError(st, "kvc_reconstruct_attend_decode")

    for step in warm:                       # warm-up: same slot, text length not advanced
        for a in step:
            layer_step(a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in timed:                      # timed: text cache grows by one token per step
        for a in step:
            layer_step(a)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    assert bool(torch.isfinite(out.float()).all()), "non-finite attention output"

    # ---- device time of the decode call, HIP events on the launch stream -------------------------
    # (second identical pass, so the event records do not perturb the wall-clock figure above)
    pairs = []
    for step in timed:
        for a in step:
            e0, e1 = ev(), ev()
            e0.record()
            layer_step(a)
            e1.record()
            pairs.append((e0, e1))
    torch.cuda.synchronize()
    call_us = sum(a.elapsed_time(b) for a, b in pairs) * 1e3 / len(pairs)

    if args.copy_probe:
        src = torch.empty(args.copy_probe << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    t_avg = w.text_len + (K + 1) / 2.0      # rows attended, new token included
    abytes = algorithmic_bytes(w, m, t_avg)
    achieved = abytes / (call_us * 1e-6) / 1e9
    traffic = read_traffic()
    res = {
        "metric": "decode attention steps/s + achieved HBM GB/s (% peak) at 60% vision-KV compression",
        "value": K / wall, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, B=%d, %dq/%dkv heads, d=%d, %d images x %d vision "
                               "tokens, text %d->%d, compression %.0f%% (m=%d)"
                               % (w.name, L, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                  w.n_images, w.n_img_tokens, w.text_len, w.text_len + K,
                                  100 * w.compression, m),
                   "kernels": "generic" if args.generic else "mfma"},
        "layer_steps_per_s": K * L / wall,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic["bytes_per_call"] if traffic else None,
                     "kernel": "kvc_reconstruct_attend_decode (fa_scores + fb_expand + fc_output)",
                     "algorithmic_bytes_per_launch": abytes, "us_per_launch": call_us},
        "compress": {"ms_per_layer": comp_ms / L,
                     "tflops": 2.0 * w.batch * w.n_kv_heads * w.n_images * m * w.n_img_tokens
                     * w.head_dim / (comp_ms / L * 1e-3) / 1e12},
    }

    # ---- CPU oracle on the host cores, bounded sample: one layer-step of layer 0 -------------------
    if not args.no_cpu_baseline:
        from oracle import kvc_oracle as orc

        def f64(x):
            return x.detach().cpu().to(torch.float64).numpy()
        Lr = layers[0]
        a = [f64(q_all[W, 0]), f64(Lr["Kc"]), f64(Lr["Vc"]), f64(Lr["p"]["theta"]),
             f64(Lr["p"]["U"]), f64(Lr["p"]["mu"])]
        Ktd, Vtd = f64(Lr["Kt"]).copy(), f64(Lr["Vt"]).copy()
        c0 = time.perf_counter()
        orc.reconstruct_attend_decode(a[0], a[1], a[2], a[3], a[4], a[5], w.n_img_tokens, Ktd, Vtd,
                                      w.text_len, f64(kn_all[W, 0]), f64(vn_all[W, 0]))
        c1 = time.perf_counter()
        res["cpu_baseline"] = {"value": 1.0 / ((c1 - c0) * L), "unit": "steps/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": "one decode step of layer 0 of %d (all batch elements, "
                                         "heads and images), %.2f s; steps/s = 1/(L x that)"
                                         % (L, c1 - c0)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
