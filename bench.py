#!/usr/bin/env python3
"""Benchmark of the Winograd F(m x m, 3 x 3) forward path on one MI355X.

A step is one forward pass of the 13 VGG-16 3x3 convolution layers (shapes of Table 3 of
Lavin & Gray) on synthetic N(0,1) data and He-scaled filters resident in HBM: conv1.1 through
the direct kernel, every other layer through wino_conv2d_fwd_ex (filter transform, input
transform, batched multiply, inverse transform).  The headline value is effective TFLOP/s as
the paper defines it (Section 7): direct-convolution flops divided by run time.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 64] [--dtype f32]

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (the transform-domain multiply) against the MFMA peak,
                timed per launch with HIP events in a separate pass over the same launches;
  stages        per-stage achieved GB/s (transforms) and TFLOP/s (multiply), per layer;
  n1            the same stack at batch 1 (the latency case of the paper's Table 5);
  bwd_data      the input gradient of the same layers (Section 4.2: same algorithm, rotated filters);
  bwd_filter    the filter gradient of the same layers (Section 4.2, Eq. (14): F(3x3,2x2));
  f6x6          the same layers through F(6x6,3x3) (Section 4.3), per layer, next to the headline algorithm;
  cpu_baseline  the fp64 CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm_GBs": 8000.0, "mfma_f32_TFs": 157.3, "mfma_f16_TFs": 2500.0}
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see
# profiles/); keyed by (workload, kernel).  None until measured for a workload.
MEASURED_TRAFFIC = {
    # profiles/vgg16_n64_fp32_hbm_traffic.md: 269.0 MB read + 265.5 MB written per launch (algorithmic 511.1 MB)
    ("vgg16_3x3_conv_stack_N64_f32", "gemm_f32_kernel<128, 128, 2, 2, 16>"): 534.5e6,
}
# Titan X (Maxwell) numbers of the paper, F(2x2,3x3), VGG network E (Tables 5 and 6): context only.
PAPER_TITANX = {"fp32": {1: 7.03, 64: 9.37}, "fp16": {1: 7.06, 64: 10.28}}


def direct_flops(N, C, H, W, K, R=3, S=3):
    """Flops of Eq. (1) with H x W outputs: 2 per multiply-add (the convention of Table 3)."""
    return 2 * N * K * C * R * S * H * W


def choose_m(HW, policy):
    """'auto': the algorithms the N=64 workload names -- F(4x4,3x3) where 4 divides the image, else F(2x2,3x3).
    'auto_n1' (the batch-1 stack, for which the workload names no algorithm) takes F(2x2,3x3) for images of 28x28
    and below as well: with a handful of tiles the layer is bound by the transformed filters, which are 2.25x
    smaller.  Or a fixed m."""
    if policy == "auto":
        return 4 if HW % 4 == 0 else 2
    if policy == "auto_n1":
        return 4 if (HW % 4 == 0 and HW > 28) else 2
    return int(policy)


class Layer:
    pass


def make_layers(N, np_dtype, policy, config_idx):
    import torch
    import paper_1509_09308_amd as w
    from paper_1509_09308_amd import synth
    layers = []
    for li, (name, C, HW, K) in enumerate(synth.VGG16_LAYERS):
        L = Layer()
        L.name, L.C, L.HW, L.K, L.N = name, C, HW, K, N
        L.direct = C < 16
        L.m = None if L.direct else choose_m(HW, policy)
        D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(config_idx, li), dtype=np_dtype)
        L.D_host, L.G_host = D, G
        L.D, L.G = torch.from_numpy(D).cuda(), torch.from_numpy(G).cuda()
        L.Y = torch.empty((N, K, HW, HW), dtype=torch.float32 if not L.direct else L.D.dtype, device="cuda")
        L.flops = direct_flops(N, C, HW, HW, K)
        if not L.direct:
            L.dt = w.WINO_F32 if L.D.dtype == torch.float32 else w.WINO_F16
            L.P = w.wino_num_tiles(N, HW, HW, 1, L.m)
            L.ws_bytes = w.wino_workspace_bytes(N, C, HW, HW, K, 1, L.m, L.dt)
            L.variant = w.wino_conv2d_variant(N, C, HW, HW, K, 1, L.m, L.dt)
        layers.append(L)
    return layers


def run_step(w, layers, ws):
    for L in layers:
        if L.direct:
            w.direct_conv2d_fwd(L.D, L.G, pad=1, Y=L.Y)
        else:
            w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=L.m, Y=L.Y, workspace=ws)


def time_steps(torch, w, layers, ws, steps, warmup):
    for _ in range(warmup):
        run_step(w, layers, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step(w, layers, ws)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_layers(torch, w, layers, ws, steps):
    """Per-layer time of the same calls, HIP events on the launch stream."""
    out = []
    for L in layers:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        run_step(w, [L], ws)
        ev[0].record()
        for i in range(steps):
            run_step(w, [L], ws)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
        out.append(sum(ts) / len(ts))
    return out


def time_stages(torch, w, layers, ws, steps):
    """Second pass over the same launches, one kernel at a time, each bracketed by HIP events on
    the stream the kernels run on.  A layer that wino_conv2d_fwd_ex runs through the one-kernel
    path is timed as {filter transform, fused kernel}; the others as the four stage kernels.
    Returns per-layer dictionaries (times in ms)."""
    res = []
    es = lambda: torch.cuda.Event(enable_timing=True)
    for L in layers:
        if L.direct:
            res.append(None)
            continue
        a2 = (L.m + 2) ** 2
        s = 4 if L.dt == w.WINO_F32 else 2
        Kp, Cp, Pp = w.wino_padded_dims(L.K, L.C, L.P, L.m, L.dt)
        U = w.alloc_u(L.K, L.C, L.m, L.dt)
        st = {"variant": L.variant, "gemm_flops": 2 * a2 * L.K * L.C * L.P}
        if L.variant == w.FLAG_FUSED:
            # fp32: the call transforms the filters itself (into the channel-pair order its kernel reads), so
            # the filter transform (a 5-10 us launch) cannot be separated and is inside "fused";
            # fp16 storage: pre-transformed filters are passed and timed on their own
            acc = {"filter": 0.0, "fused": 0.0}
            f32 = L.dt == w.WINO_F32
            for it in range(steps + 1):
                e = [es() for _ in range(3)]
                e[0].record()
                if not f32:
                    w.wino_filter_transform(L.G, L.m, U=U)
                e[1].record()
                if f32:
                    w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=L.m, Y=L.Y, workspace=ws, flags=w.FLAG_FUSED)
                else:
                    w.wino_conv2d_fwd_ex(L.D, U=U, K=L.K, pad=1, m=L.m, Y=L.Y, workspace=ws, flags=w.FLAG_FUSED)
                e[2].record()
                torch.cuda.synchronize()
                if it:
                    for j, k in enumerate(("filter", "fused")):
                        acc[k] += e[j].elapsed_time(e[j + 1]) / steps
            st.update(acc)
            if f32:
                del st["filter"]
            st["kernel"] = "fused_pair_kernel" if f32 else "fused_f16_kernel"
            st["bytes"] = {"filter": 9 * L.K * L.C * s + a2 * L.K * L.C * s,
                           "fused": L.N * L.C * L.HW * L.HW * s + a2 * L.K * L.C * s + L.N * L.K * L.HW * L.HW * 4}
        else:
            V = w.alloc_v(L.C, L.P, L.m, L.dt)
            M = w.alloc_m(L.K, L.P, L.m)
            acc = {"filter": 0.0, "input": 0.0, "gemm": 0.0, "output": 0.0}
            for it in range(steps + 1):
                e = [es() for _ in range(5)]
                e[0].record()
                w.wino_filter_transform(L.G, L.m, U=U)
                e[1].record()
                w.wino_input_transform(L.D, 1, L.m, V=V)
                e[2].record()
                w.wino_batched_gemm(U, V, L.K, L.C, L.P, L.m, M=M)
                e[3].record()
                w.wino_output_transform(M, L.N, L.K, L.HW, L.HW, 1, L.m, Y=L.Y)
                e[4].record()
                torch.cuda.synchronize()
                if it:
                    for j, k in enumerate(("filter", "input", "gemm", "output")):
                        acc[k] += e[j].elapsed_time(e[j + 1]) / steps
            st.update(acc)
            st["bytes"] = {
                "filter": 9 * L.K * L.C * s + a2 * L.K * L.C * s,
                "input": L.N * L.C * L.HW * L.HW * s + a2 * L.C * L.P * s,
                "output": a2 * L.K * L.P * 4 + L.N * L.K * L.HW * L.HW * 4,
                "gemm": a2 * (L.K * L.C + L.C * L.P) * s + a2 * L.K * L.P * 4,   # U and V read, M (fp32) written
            }
            bm, bn, _ = w.wino_gemm_launch_shape(L.K, L.C, L.P, L.m, L.dt)
            tile = "%d, %d" % (bm, bn)
            st["kernel"] = ("gemm_f32_kernel<%s, 2, 2, 16>" % tile) if L.dt == w.WINO_F32 else ("gemm_f16_kernel<%s>" % tile)
            del V, M
        res.append(st)
        del U
    return res


def time_bwd_data(torch, w, layers, ws_bytes, steps):
    """Input gradient (Section 4.2 of the paper) of the 12 layers that need one (not the first):
    the error tensor is the layer's output buffer, same algorithm choice as the forward pass."""
    todo = [L for L in layers if not L.direct]
    need = max(w.wino_workspace_bytes(L.N, L.K, L.HW, L.HW, L.C, 1, L.m, L.dt) for L in todo)
    ws = torch.empty(max(need, ws_bytes), dtype=torch.uint8, device="cuda")
    grads = [torch.empty_like(L.D, dtype=torch.float32) for L in todo]

    def step():
        for L, dD in zip(todo, grads):
            w.wino_conv2d_bwd_data(L.Y.to(L.D.dtype) if L.Y.dtype != L.D.dtype else L.Y, G=L.G, pad=1, m=L.m, dD=dD,
                                   workspace=ws)
    if any(L.Y.dtype != L.D.dtype for L in todo):
        return None   # fp16 storage keeps fp32 outputs: no resident fp16 error tensor to time
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    flops = sum(L.flops for L in todo)
    return {"eff_tflops": flops / sec / 1e12, "ms_per_step": sec * 1e3, "layers": len(todo),
            "note": "conv1.1 needs no input gradient; effective flops as for the forward pass"}


def time_bwd_filter(torch, w, layers, steps):
    """Filter gradient (Section 4.2, Eq. (14): F(3x3,2x2)) of all 13 layers, fp32: D is the layer's
    input, the error tensor its output buffer."""
    if any(L.D.dtype != torch.float32 or L.Y.dtype != torch.float32 for L in layers):
        return None
    need = max(w.wino_bwd_filter_workspace_bytes(L.N, L.C, L.HW, L.HW, L.K) for L in layers)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    grads = [torch.empty_like(L.G) for L in layers]
    per = []
    for L, dG in zip(layers, grads):
        for _ in range(2):
            w.wino_conv2d_bwd_filter(L.D, L.Y, pad=1, dG=dG, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.wino_conv2d_bwd_filter(L.D, L.Y, pad=1, dG=dG, workspace=ws)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        per.append({"layer": L.name, "ms": sec * 1e3, "eff_tflops": L.flops / sec / 1e12})
    sec = sum(p["ms"] for p in per) / 1e3
    return {"eff_tflops": sum(L.flops for L in layers) / sec / 1e12, "ms_per_step": sec * 1e3, "layers": len(layers),
            "per_layer": per, "note": "effective flops as for the forward pass"}


def time_f6x6(torch, w, layers, layer_ms, steps):
    """The same layers through F(6x6,3x3) (Section 4.3 mentions it; 5.06x fewer multiplications, edge
    tiles zero-filled where 6 does not divide the image), fp32, four separate stages."""
    todo = [(L, t) for L, t in zip(layers, layer_ms) if not L.direct]
    if any(L.D.dtype != torch.float32 for L, _ in todo):
        return None
    ws = torch.empty(max(w.wino_workspace_bytes(L.N, L.C, L.HW, L.HW, L.K, 1, 6, L.dt) for L, _ in todo),
                     dtype=torch.uint8, device="cuda")
    per, best_ms = [], sum(t for L, t in zip(layers, layer_ms) if L.direct)
    for L, base in todo:
        for _ in range(2):
            w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=6, Y=L.Y, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=6, Y=L.Y, workspace=ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        per.append({"layer": L.name, "ms": ms, "eff_tflops": L.flops / ms / 1e9, "headline_m": L.m, "headline_ms": base})
        best_ms += min(ms, base)
    tot = sum(p["ms"] for p in per)
    return {"eff_tflops": sum(L.flops for L, _ in todo) / tot / 1e9, "ms_per_step": tot, "layers": len(per),
            "per_layer": per,
            "best_of_per_layer": {"ms_per_step": best_ms, "eff_tflops": sum(L.flops for L in layers) / best_ms / 1e9,
                                  "note": "all 13 layers, each with the faster of its headline algorithm and "
                                          "F(6x6,3x3); context only, not the headline policy"}}


def time_all_f4x4(torch, w, layers, steps, warmup):
    """The same stack with F(4x4,3x3) for the layers whose images 4 does not divide as well (the 14x14 ones: 16 tiles
    of 36 products per image and channel instead of 49 of 16, edge tiles reaching past the image).  Not the algorithm
    the workload names for them, so it is reported beside the headline, not as it."""
    changed = [L for L in layers if not L.direct and L.m != 4]
    if not changed:
        return None
    saved = [(L.m, L.P, L.ws_bytes) for L in changed]
    for L in changed:
        L.m = 4
        L.P = w.wino_num_tiles(L.N, L.HW, L.HW, 1, 4)
        L.ws_bytes = w.wino_workspace_bytes(L.N, L.C, L.HW, L.HW, L.K, 1, 4, L.dt)
    ws = torch.empty(max(L.ws_bytes for L in layers if not L.direct), dtype=torch.uint8, device="cuda")
    sec = time_steps(torch, w, layers, ws, steps, warmup)
    ms = time_layers(torch, w, changed, ws, steps)
    res = {"ms_per_step": sec * 1e3, "eff_tflops": sum(L.flops for L in layers) / sec / 1e12,
           "layers_changed": [{"layer": L.name, "ms": t, "eff_tflops": L.flops / t / 1e9} for L, t in zip(changed, ms)]}
    for L, (m, P, wsb) in zip(changed, saved):
        L.m, L.P, L.ws_bytes = m, P, wsb
    return res


def time_one_launch(torch, w, layers, steps, warmup):
    """The batch-1 stack with every Winograd layer as ONE kernel launch: F(2x2,3x3) with the filter
    transform inside the kernel (Section 6 of the paper, the variant without separately transformed
    filters); conv1.1 stays direct."""
    ws = torch.empty(max(w.wino_workspace_bytes(L.N, L.C, L.HW, L.HW, L.K, 1, 2, L.dt) for L in layers if not L.direct),
                     dtype=torch.uint8, device="cuda")

    def step():
        for L in layers:
            if L.direct:
                w.direct_conv2d_fwd(L.D, L.G, pad=1, Y=L.Y)
            else:
                w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=2, Y=L.Y, workspace=ws, flags=w.FLAG_ONE_LAUNCH)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t = (time.perf_counter() - t0) / steps
    return {"ms_per_step": t * 1e3, "eff_tflops": sum(L.flops for L in layers) / t / 1e12, "launches_per_step": len(layers)}


def time_graph(torch, w, layers, ws, steps):
    """The whole step captured once in a HIP graph and replayed: removes the host's launch work, not the
    GPU's per-kernel start-up and drain.  Replays alternate with eager steps and are compared with them."""
    refs = [L.Y.clone() for L in layers]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run_step(w, layers, ws)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run_step(w, layers, ws)
    torch.cuda.synchronize()
    same = True
    for _ in range(3):
        for L in layers:
            L.Y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        same = same and all(torch.equal(a, L.Y) for a, L in zip(refs, layers))
        run_step(w, layers, ws)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return {"ms_per_step": (time.perf_counter() - t0) / steps * 1e3, "replays_equal_eager": bool(same)}


def cpu_baseline(layers, budget_s=12.0, max_images=32):
    """The fp64 oracle (Eq. (1)) on the host cores over whole images of the same workload:
    image after image through all 13 layers until about `budget_s` seconds have been spent."""
    from oracle import direct
    flops, secs, imgs = 0.0, 0.0, 0
    nmax = layers[0].N
    while secs < budget_s and imgs < max_images:
        for L in layers:
            D = L.D_host[imgs % nmax:imgs % nmax + 1]
            t0 = time.perf_counter()
            direct.conv2d_fwd(D, L.G_host, pad=1)
            secs += time.perf_counter() - t0
            flops += direct_flops(1, L.C, L.HW, L.HW, L.K)
        imgs += 1
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": direct.num_threads(), "kind": "oracle",
            "images_per_sec": imgs / secs,
            "sample": "fp64 direct convolution of all 13 layers, %d image(s) of the batch of %d, %.1f s of CPU time"
                      % (imgs, nmax, secs)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--dtype", choices=["f32", "f16"], default="f32")
    ap.add_argument("--m", default="auto", help="auto | 2 | 4 | 6 (6: fp32 only)")
    ap.add_argument("--no-n1", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stages", action="store_true")
    ap.add_argument("--no-bwd", action="store_true", help="skip the input- and filter-gradient lines")
    ap.add_argument("--no-f6", action="store_true", help="skip the F(6x6,3x3) and all-F(4x4,3x3) lines")
    ap.add_argument("--graph", action="store_true",
                    help="also time the batch-1 stack captured in a HIP graph and replayed (every replay is checked "
                         "against the eager result)")
    ap.add_argument("--probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (counter calibration), then every "
                         "kernel of one step once; prints the algorithmic bytes per kernel and exits")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (batch sharding across GPUs is a design note, "
              "not built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1509_09308_amd as w
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    w.build.ensure_built()
    torch.cuda.set_device(0)
    np_dtype = np.float32 if args.dtype == "f32" else np.float16
    cfg_idx = 4 if args.dtype == "f32" else 5
    policy = args.m if args.dtype == "f32" else ("4" if args.m == "auto" else args.m)
    if args.batch == 1 and args.dtype == "f32" and policy == "auto":
        policy = "auto_n1"        # the choice the n1 line of the default run makes

    layers = make_layers(args.batch, np_dtype, policy, cfg_idx)
    ws = torch.empty(max(L.ws_bytes for L in layers if not L.direct), dtype=torch.uint8, device="cuda")
    total_flops = sum(L.flops for L in layers)

    if args.probe:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                                                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
        st = time_stages(torch, w, layers, ws, 1)
        print(json.dumps({"probe": "1 GiB copy, then each kernel of one step twice (warm-up + timed)",
                          "layers": [{"layer": L.name, "kernel": x["kernel"], "flops": x["gemm_flops"],
                                      "bytes": x["bytes"]} for L, x in zip(layers, st) if x]}))
        return
    sec = time_steps(torch, w, layers, ws, args.steps, args.warmup)
    value = total_flops / sec / 1e12

    layer_ms = time_layers(torch, w, layers, ws, max(3, args.steps))
    # the same per-layer times re-weighted with the depths of VGG network E (Table 3 of the paper)
    from paper_1509_09308_amd import synth
    shape = lambda L: (L.C, L.HW, L.K)
    count16 = {}
    for L in layers:
        count16[shape(L)] = count16.get(shape(L), 0) + 1
    wE = [synth.VGG_E_DEPTH[shape(L)] / count16[shape(L)] for L in layers]
    e_flops = sum(x * L.flops for x, L in zip(wE, layers))
    e_ms = sum(x * t for x, t in zip(wE, layer_ms))

    out = {
        "metric": "effective conv TFLOPS, VGG-16 3x3 conv stack forward, N=%d, 1 GPU" % args.batch,
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "vgg16_3x3_conv_stack_N%d_%s" % (args.batch, args.dtype), "batch": args.batch,
                   "layers": 13, "algorithm": "F(4x4,3x3) where 4 divides H, else F(2x2,3x3); conv1.1 direct"
                   if policy == "auto" else "F(4x4,3x3) for images of 56x56 and more, else F(2x2,3x3); conv1.1 direct"
                   if policy == "auto_n1" else "F(%sx%s,3x3); conv1.1 direct" % (policy, policy),
                   "filter_transform": "inside the timed step"},
        "images_per_sec": args.batch / sec,
        "direct_gflop_per_step": total_flops / 1e9,
        "per_layer": [{"layer": L.name, "m": L.m, "ms": t, "eff_tflops": L.flops / t / 1e9}
                      for L, t in zip(layers, layer_ms)],
        "vgg_e_weighted": {"eff_tflops": e_flops / e_ms / 1e9, "ms": e_ms,
                           "paper_titanx_f2x2_tflops": PAPER_TITANX["fp32" if args.dtype == "f32" else "fp16"].get(args.batch)},
    }

    if not args.no_stages:
        stages = time_stages(torch, w, layers, ws, max(3, args.steps))
        rows, dom = [], {}
        hb, hms = 0.0, 0.0
        for L, st in zip(layers, stages):
            if st is None:
                continue
            main = "fused" if st["variant"] == w.FLAG_FUSED else "gemm"
            row = {"layer": L.name, "m": L.m, "variant": "fused" if main == "fused" else "unfused",
                   "kernel": st["kernel"], "kernel_ms": st[main], "kernel_tflops": st["gemm_flops"] / st[main] / 1e9}
            for k in ("filter", "input", "output"):
                if k in st:
                    row[k + "_ms"] = st[k]
                    row[k + "_GBs"] = st["bytes"][k] / st[k] / 1e6
                    if k != "filter":
                        hb += st["bytes"][k]
                        hms += st[k]
            rows.append(row)
            d = dom.setdefault(st["kernel"], {"flops": 0.0, "ms": 0.0, "launches": 0, "bytes": 0.0})
            d["flops"] += st["gemm_flops"]
            d["bytes"] += st["bytes"].get("gemm", 0.0) if main == "gemm" else 0.0
            d["ms"] += st[main]
            d["launches"] += 1
        out["stages"] = rows
        peak = PEAK["mfma_f32_TFs"] if args.dtype == "f32" else PEAK["mfma_f16_TFs"]
        out["kernels"] = {k: {"launches_per_step": d["launches"], "avg_launch_ms": d["ms"] / d["launches"],
                              "tflops": d["flops"] / d["ms"] / 1e9, "frac_of_mfma_peak": d["flops"] / d["ms"] / 1e9 / peak}
                          for k, d in dom.items()}
        if dom:
            name, d = max(dom.items(), key=lambda kv: kv[1]["ms"])
            ach = d["flops"] / d["ms"] / 1e9
            out["roofline"] = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                               "traffic": MEASURED_TRAFFIC.get((out["config"]["workload"], name)), "kernel": name,
                               "launches_per_step": d["launches"], "avg_launch_ms": d["ms"] / d["launches"],
                               "flops_per_launch": d["flops"] / d["launches"]}
            # a multiply whose flops per byte fall below the machine balance (peak flops / peak bytes) is
            # bound by HBM, not by the matrix cores: the fp16-storage multiply (fp32 M written out) is
            if d["bytes"] > 0 and d["flops"] / d["bytes"] < peak * 1e12 / (PEAK["hbm_GBs"] * 1e9):
                gbs = d["bytes"] / d["ms"] / 1e6
                out["roofline"].update({"bound": "hbm", "achieved": gbs, "peak": PEAK["hbm_GBs"], "unit": "GB/s",
                                        "frac": gbs / PEAK["hbm_GBs"], "bytes_per_launch": d["bytes"] / d["launches"],
                                        "mfma_tflops": ach, "flops_per_byte": d["flops"] / d["bytes"]})
        if hms > 0:
            out["transform_roofline"] = {"bound": "hbm", "achieved": hb / hms / 1e6, "peak": PEAK["hbm_GBs"],
                                         "unit": "GB/s", "frac": hb / hms / 1e6 / PEAK["hbm_GBs"],
                                         "kernels": "input_transform + output_transform of the unfused layers"}

    if not args.no_bwd:
        bd = time_bwd_data(torch, w, layers, ws.numel(), max(3, args.steps // 2))
        if bd:
            out["bwd_data"] = bd
        bf = time_bwd_filter(torch, w, layers, max(3, args.steps // 2))
        if bf:
            out["bwd_filter"] = bf
    if not args.no_f6 and policy == "auto" and args.dtype == "f32":
        f4 = time_all_f4x4(torch, w, layers, args.steps, args.warmup)
        if f4:
            out["all_f4x4"] = f4
    if not args.no_f6 and policy == "auto":
        f6 = time_f6x6(torch, w, layers, layer_ms, max(3, args.steps // 2))
        if f6:
            out["f6x6"] = f6
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers)
    if args.batch == 1 and args.dtype == "f32":
        out["one_launch_per_layer"] = time_one_launch(torch, w, layers, max(args.steps, 20), max(args.warmup, 5))
    if not args.no_n1 and args.batch != 1:
        del layers, ws
        torch.cuda.empty_cache()
        l1 = make_layers(1, np_dtype, policy if (args.dtype == "f16" or policy != "auto") else "auto_n1", 3)
        ws1 = torch.empty(max(L.ws_bytes for L in l1 if not L.direct), dtype=torch.uint8, device="cuda")
        s1 = time_steps(torch, w, l1, ws1, max(args.steps, 20), max(args.warmup, 5))
        f1 = sum(L.flops for L in l1)
        out["n1"] = {"eff_tflops": f1 / s1 / 1e12, "ms_per_step": s1 * 1e3, "images_per_sec": 1.0 / s1,
                     "algorithm": {L.name: ("direct" if L.direct else "F(%dx%d,3x3)" % (L.m, L.m)) for L in l1}}
        if args.dtype == "f32":
            out["n1"]["one_launch_per_layer"] = time_one_launch(torch, w, l1, max(args.steps, 20), max(args.warmup, 5))
        if args.graph:
            out["n1"]["hip_graph"] = time_graph(torch, w, l1, ws1, max(args.steps, 20))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
