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


def compress_report(w, ms, ms_per_layer, b=2):
    """One kvc_compress call per layer (event pair around each call): time, matrix-core rate and the
    HBM bytes it must move (V block and the retained key rows read, both capsule halves written, U,
    mu and the mask read once) against the HBM peak."""
    m = sum(ms) / len(ms)
    units = w.batch * w.n_kv_heads * w.n_images
    flops = 2.0 * units * m * w.n_img_tokens * w.head_dim
    nbytes = units * (w.n_img_tokens + 3 * m) * w.head_dim * b + w.n_kv_heads * (m * w.n_img_tokens + w.head_dim) * b + 4 * m
    sec = ms_per_layer * 1e-3
    return {"ms_per_layer": ms_per_layer, "tflops": flops / sec / 1e12,
            "algorithmic_bytes_per_layer": nbytes, "achieved_gbs": nbytes / sec / 1e9,
            "hbm_frac": nbytes / sec / 1e9 / HBM_PEAK_GBS}


def read_traffic(workload, compression, kernels, pyramid):
    """Measured HBM bytes per decode call from the committed rocprofv3 counter summary; None unless
    that summary was taken on this very workload, compression and kernel path."""
    path = os.path.join(ROOT, "profiles", "decode_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("workload_name") != workload or abs(t.get("compression", -1.0) - compression) > 1e-9 or pyramid:
        return None
    if t.get("kernels") == kernels:
        return t
    return t.get("other_paths", {}).get(kernels)       # the same workload on the library's other kernel path


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="qwen2vl")
    ap.add_argument("--compression", type=float, default=0.6)
    ap.add_argument("--pyramid", action="store_true",
                    help="per-layer schedule: compression ramps linearly over the layers from "
                         "(c - 0.2) to (c + 0.2), averaging --compression")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--generic", action="store_true", help="force the scalar kernels")
    ap.add_argument("--no-packed-theta", action="store_true",
                    help="do not pass the packed forms of theta and U: every call takes the four-kernel form")
    ap.add_argument("--no-full-baseline", action="store_true",
                    help="skip the full-cache (All KV) decode that is timed beside the capsule path")
    ap.add_argument("--read-probe", type=int, default=4, metavar="GiB",
                    help="time a plain streaming read over this many GiB and report it as "
                         "roofline.measured_read_ceiling (GB/s); 0 skips it")
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
    if args.batch:
        w = w.with_(batch=args.batch)
    K, W = args.steps, args.warmup
    L = w.layers
    # compressed length per layer: one value, or a pyramid schedule (Sec. 3.2: per-layer budgets
    # whose average is the quoted rate; the schedule itself is not printed, a linear ramp is used)
    if args.pyramid and L > 1:
        rates = [min(0.99, max(0.0, w.compression - 0.2 + 0.4 * l / (L - 1))) for l in range(L)]
    else:
        rates = [w.compression] * L
    ms = [kv.kvc_compressed_len(w.n_img_tokens, c) for c in rates]
    m = ms[0]
    cap = w.text_len + K
    shapes = [kv.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_img_tokens,
                            w.n_images, ml, w.torch_dtype) for ml in ms]
    big = max(range(L), key=lambda l: kv.kvc_workspace_bytes(shapes[l], cap))
    ws = kv.new_workspace(shapes[big], cap, dev)
    dt = w.torch_dtype

    # ---- build the per-layer state on the device: parameters, capsule, text cache ------------
    # Workloads with few layers get several copies of every layer's buffers, used in turn from step
    # to step, so that at least 8 distinct working sets pass before one is revisited (otherwise the
    # 256 MB memory-side cache would serve a single layer's capsule).
    copies = 1 if L >= 8 else -(-8 // L)
    layers = []
    ev = lambda: torch.cuda.Event(enable_timing=True)
    comp_ms = 0.0
    for lc in range(L * copies):
        l = lc % L
        shape, cshape = shapes[l], (w.batch, w.n_kv_heads, w.n_images, ms[l], w.head_dim)
        p = synth.make_params(w, ms[l], l, device=dev)
        # theta and U re-tiled once at load time (kvc_pack_theta, kvc_pack_u): calls whose shape has a one-pass kernel use them
        if not args.generic and not args.no_packed_theta:
            p["theta_packed"] = kv.kvc_pack_theta(shape, p["theta"])
            p["U_packed"] = kv.kvc_pack_u(shape, p["U"])
        params = kv.make_params(p["key_idx"], p["theta"], p["U"], p["mu"], p.get("theta_packed"), p.get("U_packed"))
        Kp, Vp = synth.make_prefill_kv(w, l, 0, 0, device=dev)
        Kc = torch.empty(cshape, dtype=dt, device=dev)
        Vc = torch.empty(cshape, dtype=dt, device=dev)
        e0, e1 = ev(), ev()
        if lc == 0:     # untimed first call (module load)
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
    vp = ctypes.c_void_p

    def marshal(s, l, t):
        Lr = layers[(s % copies) * L + l]
        return (ctypes.byref(shapes[l]), ctypes.byref(Lr["params"]), vp(q_all[s, l].data_ptr()),
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

    stream_calls0 = kv.lib().kvc_dev_stream_calls()
    for step in warm:                       # warm-up: same slot, text length not advanced
        for a in step:
            layer_step(a)
    # the timed region is also bracketed by one pair of HIP events on the launch stream: the device
    # time of the K x L calls, launch gaps between them included, with nothing recorded in between
    ev_beg, ev_end = ev(), ev()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev_beg.record()
    for step in timed:                      # timed: text cache grows by one token per step
        for a in step:
            layer_step(a)
    ev_end.record()
    t_issued = time.perf_counter()          # the host has handed over every call; the device is still working
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    assert bool(torch.isfinite(out.float()).all()), "non-finite attention output"
    stream_share = (kv.lib().kvc_dev_stream_calls() - stream_calls0) / float((W + K) * L)
    kernels = "generic" if args.generic else "mfma-one-pass" if stream_share == 1.0 else \
        "mfma" if stream_share == 0.0 else "mfma (one-pass kernel for %.0f%% of the calls)" % (100 * stream_share)
    call_us = ev_beg.elapsed_time(ev_end) * 1e3 / (K * L)

    # second identical pass with an event pair around every single call (each pair adds about 2 us
    # of stream work, so this figure is an upper bound of the per-call device time)
    pairs = []
    for step in timed:
        for a in step:
            e0, e1 = ev(), ev()
            e0.record()
            layer_step(a)
            e1.record()
            pairs.append((e0, e1))
    torch.cuda.synchronize()
    call_us_pairs = sum(a.elapsed_time(b) for a, b in pairs) * 1e3 / len(pairs)

    # ---- the same decode step without KVCapsule: full-cache attention over N + t rows ------------
    # (the "All KV" comparison point of the paper's efficiency analysis), every layer with its own
    # cache, same number of steps, text growing by one token per step
    full = None
    if not args.no_full_baseline and not args.generic:
        del layers
        torch.cuda.empty_cache()
        N = w.n_images * w.n_img_tokens
        fws = torch.empty(kv.kvc_attend_full_workspace_bytes(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                                             dt, N + cap) + 256, dtype=torch.uint8, device=dev)
        caches = [synth.make_prefill_kv(w, lc % L, 0, cap, device=dev) for lc in range(L * copies)]
        fwp, fwb = kv._ws(fws)
        ffn = kv.lib().kvc_attend_full_decode
        code = kv._dtype_code(dt)

        def fmarshal(s, l, t):
            Kf, Vf = caches[(s % copies) * L + l]
            return (w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, code, vp(q_all[s, l].data_ptr()),
                    vp(Kf.data_ptr()), vp(Vf.data_ptr()), Kf.stride(0), Kf.stride(1), Kf.stride(2), N + t,
                    N + cap, vp(kn_all[s, l].data_ptr()), vp(vn_all[s, l].data_ptr()), ctypes.c_float(0.0),
                    vp(out[l].data_ptr()), None, fwp, fwb, stream)

        fwarm = [[fmarshal(s, l, w.text_len) for l in range(L)] for s in range(W)]
        ftimed = [[fmarshal(W + s, l, w.text_len + s) for l in range(L)] for s in range(K)]
        for step in fwarm:
            for a in step:
                if ffn(*a) != kv.KVC_OK:
                    raise kv.KvcError(-1, "kvc_attend_full_decode")
        f_beg, f_end = ev(), ev()
        torch.cuda.synchronize()
        f_beg.record()
        for step in ftimed:
            for a in step:
                ffn(*a)
        f_end.record()
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out.float()).all()), "non-finite full-cache attention output"
        full_us = f_beg.elapsed_time(f_end) * 1e3 / (K * L)
        t_avg_f = w.text_len + (K + 1) / 2.0
        fbytes = 2 * w.batch * w.n_kv_heads * (N + t_avg_f) * w.head_dim * 2 + 2 * w.batch * w.n_q_heads * w.head_dim * 2
        full = {"us_per_call": full_us, "algorithmic_bytes_per_call": fbytes,
                "achieved_gbs": fbytes / (full_us * 1e-6) / 1e9,
                "frac_of_hbm_peak": fbytes / (full_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "capsule_us_per_call": call_us, "capsule_speedup": full_us / call_us,
                "what": "kvc_attend_full_decode over the uncompressed cache (%d vision + text rows), "
                        "same batch, heads, steps and stream" % N}
        del caches

    if args.copy_probe:
        src = torch.empty(args.copy_probe << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    read_ceiling = None
    if args.read_probe:
        # the library's plain read kernel over a buffer far larger than every cache
        buf = torch.ones((args.read_probe << 30) // 4, dtype=torch.int32, device=dev)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        kv.kvc_probe_read(buf, sink)
        best = 0.0
        for _ in range(5):
            e0, e1 = ev(), ev()
            e0.record()
            kv.kvc_probe_read(buf, sink)
            e1.record()
            e1.synchronize()
            best = max(best, buf.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        read_ceiling = best
        del buf

    t_avg = w.text_len + (K + 1) / 2.0      # rows attended, new token included
    abytes = sum(algorithmic_bytes(w, ml, t_avg) for ml in ms) / L        # mean over the layers
    achieved = abytes / (call_us * 1e-6) / 1e9
    traffic = read_traffic(w.name, w.compression, kernels, args.pyramid)
    res = {
        "metric": "decode attention steps/s + achieved HBM GB/s (% peak) at 60% vision-KV compression",
        "value": K / wall, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, B=%d, %dq/%dkv heads, d=%d, %d images x %d vision "
                               "tokens, text %d->%d, compression %.0f%% (%s)"
                               % (w.name, L, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                  w.n_images, w.n_img_tokens, w.text_len, w.text_len + K,
                                  100 * w.compression,
                                  "m=%d" % m if len(set(ms)) == 1 else
                                  "pyramid m=%d..%d, mean %.1f" % (max(ms), min(ms), sum(ms) / L)),
                   "kernels": kernels, "buffer_copies": copies,
                   "params": "theta, U as given plus their packed forms (kvc_pack_theta, kvc_pack_u, made once at load "
                             "time)" if not (args.generic or args.no_packed_theta) else "theta, U as given"},
        "layer_steps_per_s": K * L / wall,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic["bytes_per_call"] if traffic else None,
                     "kernel": "kvc_reconstruct_attend_decode (kernels fs_stream, fs_finalize where the one-pass form "
                               "serves the call; fab_fused, fc_fused, fd_finalize_few otherwise; the scalar kernels "
                               "with --generic)",
                     "algorithmic_bytes_per_launch": abytes, "us_per_launch": call_us,
                     "us_per_launch_event_pair_each": call_us_pairs,
                     "host_us_per_launch": (t_issued - t0) * 1e6 / (K * L),
                     "measured_read_ceiling": read_ceiling},
        "compress": compress_report(w, ms, comp_ms / (L * copies)),
    }

    if full:
        res["full_kv_baseline"] = full

    # ---- CPU oracle on the host cores, bounded sample of the same workload -----------------------
    # Inputs are host-made synthetic arrays of the workload's shapes (nothing the GPU path produced):
    # the oracle's time depends on shapes only.  Layer-steps are repeated until about 12 s of CPU
    # work have been timed.
    if not args.no_cpu_baseline:
        import numpy as np

        from oracle import kvc_oracle as orc

        rng = np.random.default_rng(synth.BASE_SEED + 7)
        hp = synth.make_params(w, m, 0, device="cpu")
        f64 = lambda x: x.detach().cpu().to(torch.float64).numpy()
        cs = (w.batch, w.n_kv_heads, w.n_images, m, w.head_dim)
        qh = rng.standard_normal((w.batch, w.n_q_heads, w.head_dim))
        Kch, Vch = rng.standard_normal(cs), rng.standard_normal(cs)
        Kth = rng.standard_normal((w.batch, w.n_kv_heads, cap, w.head_dim))
        Vth = rng.standard_normal((w.batch, w.n_kv_heads, cap, w.head_dim))
        knh = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim))
        vnh = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim))
        th, Uh, muh = f64(hp["theta"]), f64(hp["U"]), f64(hp["mu"])
        times = []
        while sum(times) < 12.0 and len(times) < 4 * L:
            c0 = time.perf_counter()
            orc.reconstruct_attend_decode(qh, Kch, Vch, th, Uh, muh, w.n_img_tokens, Kth, Vth,
                                          w.text_len, knh, vnh)
            times.append(time.perf_counter() - c0)
        per_layer = sum(times) / len(times)
        res["cpu_baseline"] = {"value": 1.0 / (per_layer * L), "unit": "steps/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": "%d layer-steps of the decode path (all batch elements, heads "
                                         "and images of one layer; %.1f s in total); steps/s = "
                                         "1 / (%d layers x mean layer-step time)"
                                         % (len(times), sum(times), L)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
