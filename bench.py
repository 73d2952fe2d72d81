#!/usr/bin/env python3
"""Benchmark of the Winograd F(m x m, 3 x 3) forward path on one MI355X.

A step is one forward pass of the 13 VGG-16 3x3 convolution layers (shapes of Table 3 of
Lavin & Gray) on synthetic N(0,1) data and He-scaled filters resident in HBM: conv1.1 through
the direct kernel, every other layer through wino_conv2d_fwd_ex (filter transform, input
transform, batched multiply, inverse transform).  The headline value is effective TFLOP/s as
the paper defines it (Section 7): direct-convolution flops divided by run time, at N=64 in fp32.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 64] [--dtype f32] [--only LEG]

Prints ONE JSON line.  Besides the contract fields it carries
  roofline            the dominant kernel (the transform-domain multiply) against the MFMA peak, timed per
                      launch with HIP events in a separate pass over the same launches;
  step_ms             mean / median / min of the step, one HIP event pair per step;
  fx                  the same step with the filters transformed ahead of it (Section 6, "FX");
  stages              per-stage GB/s (transforms: hot = same buffers again, cold = buffer sets rotated so
                      that nothing is left in the caches) and TFLOP/s (multiply), per layer;
  transform_roofline  the transforms of the four-stage layers against the HBM peak (cold);
  cfg5_f16_n32        the fp16-storage workload (N=32, F(4x4,3x3) everywhere) with its own roofline;
  n1                  the same stack at batch 1 (the latency case of the paper's Table 5) with its bound;
  cfg2, cfg1          the two single-layer workloads (512 -> 512 at 28 x 28, N=8, both algorithms; 32 -> 32 at
                      56 x 56, N=1);
  bwd_data, bwd_filter, all_f4x4, f6x6   the gradients (Section 4.2) and the other tile sizes;
  cpu_baseline        the fp64 CPU oracle timed on a bounded sample of the same workload, with the
                      GPU outputs of those images checked against it.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm_GBs": 8000.0, "mfma_f32_TFs": 157.3, "mfma_f16_TFs": 2500.0}
# HBM bytes per launch of a workload's dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# `bench.py --probe` (summaries under profiles/); keyed by (workload, kernel).  None until measured.
MEASURED_TRAFFIC = {
    # profiles/vgg16_n64_fp32_hbm_traffic.md
    ("vgg16_3x3_conv_stack_N64_f32", "fused_wide_kernel<4, false>"): 1137.0e6,     # 9 launches (algorithmic 544.5 MB)
    ("vgg16_3x3_conv_stack_N64_f32", "fused_wide_kernel<2, false>"): 303.5e6,      # 3 launches (algorithmic 68.2 MB)
    # profiles/vgg16_n32_fp16_hbm_traffic.md (algorithmic: 328.7 MB resp. 183.5 MB per launch)
    ("vgg16_3x3_conv_stack_N32_f16", "fused_f16_kernel<false, 2, float>"): 355.9e6,
    ("vgg16_3x3_conv_stack_N32_f16", "gemm_f16_kernel<128, 128>"): 187.3e6,
}
# Titan X (Maxwell) numbers of the paper, F(2x2,3x3), VGG network E (Tables 5 and 6): context only.
PAPER_TITANX = {"fp32": {1: 7.03, 64: 9.37}, "fp16": {1: 7.06, 64: 10.28}}
LEGS = ("headline", "f16", "n1", "cfg2", "cfg1")


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


def stats(ts):
    ts = sorted(ts)
    n = len(ts)
    return {"mean": sum(ts) / n, "median": ts[n // 2] if n % 2 else 0.5 * (ts[n // 2 - 1] + ts[n // 2]), "min": ts[0]}


class Layer:
    pass


def make_layers(N, np_dtype, policy, config_idx, shapes=None):
    import torch
    import paper_1509_09308_amd as w
    from paper_1509_09308_amd import synth
    layers = []
    for li, (name, C, HW, K) in enumerate(shapes or synth.VGG16_LAYERS):
        L = Layer()
        L.name, L.C, L.HW, L.K, L.N = name, C, HW, K, N
        L.direct = C < 16
        L.m = None if L.direct else choose_m(HW, policy)
        D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(config_idx, li), dtype=np_dtype)
        L.D_host, L.G_host = D, G
        L.D, L.G = torch.from_numpy(D).cuda(), torch.from_numpy(G).cuda()
        L.Y = torch.empty((N, K, HW, HW), dtype=torch.float32 if not L.direct else L.D.dtype, device="cuda")
        L.flops = direct_flops(N, C, HW, HW, K)
        L.U = None
        if not L.direct:
            L.dt = w.WINO_F32 if L.D.dtype == torch.float32 else w.WINO_F16
            L.P = w.wino_num_tiles(N, HW, HW, 1, L.m)
            L.ws_bytes = w.wino_workspace_bytes(N, C, HW, HW, K, 1, L.m, L.dt)
            L.variant = w.wino_conv2d_variant(N, C, HW, HW, K, 1, L.m, L.dt)
        layers.append(L)
    return layers


def run_step(w, layers, ws, fx=False):
    for L in layers:
        if L.direct:
            w.direct_conv2d_fwd(L.D, L.G, pad=1, Y=L.Y)
        elif fx and L.U is not None:
            w.wino_conv2d_fwd_ex(L.D, U=L.U, K=L.K, pad=1, m=L.m, Y=L.Y, workspace=ws)
        else:
            w.wino_conv2d_fwd_ex(L.D, G=L.G, pad=1, m=L.m, Y=L.Y, workspace=ws)


def time_steps(torch, w, layers, ws, steps, warmup, fx=False):
    """The contract's figure: K steps between two synchronisations, host timer."""
    for _ in range(warmup):
        run_step(w, layers, ws, fx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step(w, layers, ws, fx)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_steps_events(torch, w, layers, ws, steps, fx=False):
    """The same steps once more with a HIP event between them: mean, median and min of a step (ms)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    run_step(w, layers, ws, fx)
    ev[0].record()
    for i in range(steps):
        run_step(w, layers, ws, fx)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return stats([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])


def time_layers(torch, w, layers, ws, steps):
    """Per-layer time of the same calls, HIP events on the launch stream (mean / median / min in ms)."""
    out = []
    for L in layers:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        run_step(w, [L], ws)
        ev[0].record()
        for i in range(steps):
            run_step(w, [L], ws)
            ev[i + 1].record()
        torch.cuda.synchronize()
        out.append(stats([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]))
    return out


def time_calls(torch, calls, reps):
    """`calls` is a list of closures that launch the same kernel on different buffer sets.  They are launched
    round-robin, every launch bracketed by HIP events on the launch stream; with one set that is the hot
    figure (operands may still sit in the caches), with sets whose footprints add up to more than the
    last-level cache it is the cold one.  One untimed round first."""
    for c in calls:
        c()
    n = max(reps, len(calls))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i in range(n):
        ev[i][0].record()
        calls[i % len(calls)]()
        ev[i][1].record()
    torch.cuda.synchronize()
    return stats([a.elapsed_time(b) for a, b in ev])


COLD_BYTES = 768e6     # buffer sets are rotated until this many bytes lie between two uses of one set (3x the 256 MB cache)


def n_sets(bytes_per_set):
    return int(min(12, max(3, math.ceil(COLD_BYTES / max(bytes_per_set, 1.0)) + 1)))


def stage_plan(torch, w, L, ws, sets):
    """The kernels of one layer as separately launchable calls, on `sets` buffer sets: a list (one entry per set)
    of lists of (stage name, closure) in launch order, the algorithmic bytes per stage and the kernel's name."""
    a2 = (L.m + 2) ** 2
    s = 4 if L.dt == w.WINO_F32 else 2
    nD, nY = L.N * L.C * L.HW * L.HW * s, L.N * L.K * L.HW * L.HW * 4
    nU, nV, nM = a2 * L.K * L.C * s, a2 * L.C * L.P * s, a2 * L.K * L.P * 4
    U = w.alloc_u(L.K, L.C, L.m, L.dt)
    Ds = [L.D] + [L.D.clone() for _ in range(sets - 1)]
    Ys = [L.Y] + [torch.empty_like(L.Y) for _ in range(sets - 1)]
    plans = []
    if L.variant == w.FLAG_FUSED:
        for d, y in zip(Ds, Ys):
            plans.append([("filter", lambda: w.wino_filter_transform(L.G, L.m, U=U)),
                          ("fused", (lambda d=d, y=y: w.wino_conv2d_fwd_ex(d, U=U, K=L.K, pad=1, m=L.m, Y=y, workspace=ws,
                                                                           flags=w.FLAG_FUSED)))])
        nbytes = {"filter": 9 * L.K * L.C * s + nU, "fused": nD + nU + nY}
        cpad = "false" if L.C % 8 == 0 else "true"
        if L.dt == w.WINO_F16:
            kernel = "fused_f16_kernel<%s, %d, float>" % (cpad, 2 if L.K > 32 else 1)
        elif L.K > 32:           # 64 filters per workgroup, 16 channels per step
            kernel = "fused_wide_kernel<%d, %s>" % (L.m, "false" if L.C % 16 == 0 else "true")
        else:
            kernel = "fused_lds_kernel<%s>" % cpad
    else:
        Vs = [w.alloc_v(L.C, L.P, L.m, L.dt) for _ in range(sets)]
        Ms = [w.alloc_m(L.K, L.P, L.m) for _ in range(sets)]
        for d, v, mm, y in zip(Ds, Vs, Ms, Ys):
            plans.append([("filter", lambda: w.wino_filter_transform(L.G, L.m, U=U)),
                          ("input", (lambda d=d, v=v: w.wino_input_transform(d, 1, L.m, V=v))),
                          ("gemm", (lambda v=v, mm=mm: w.wino_batched_gemm(U, v, L.K, L.C, L.P, L.m, M=mm))),
                          ("output", (lambda mm=mm, y=y: w.wino_output_transform(mm, L.N, L.K, L.HW, L.HW, 1, L.m, Y=y)))])
        nbytes = {"filter": 9 * L.K * L.C * s + nU, "input": nD + nV, "output": nM + nY,
                  "gemm": nU + nV + nM}          # U and V read, M (fp32) written
        bm, bn, _ = w.wino_gemm_launch_shape(L.K, L.C, L.P, L.m, L.dt)
        tile = "%d, %d" % (bm, bn)
        bk = 16 if (bm, bn) == (128, 128) or L.C % 32 != 0 else 32      # slab depth the library picks for this block shape
        kernel = ("gemm_f32_kernel<%s, 2, 2, %d>" % (tile, bk)) if L.dt == w.WINO_F32 else ("gemm_f16_kernel<%s>" % tile)
    return plans, nbytes, kernel, 2 * a2 * L.K * L.C * L.P


def time_stages(torch, w, layers, ws, reps, cold=True):
    """Second pass over the same launches with a HIP event between every two kernels.

    Hot: `reps` instrumented steps -- the layers in step order, each as its separate stage kernels (a layer that
    wino_conv2d_fwd_ex runs through the one-kernel path as {filter transform, fused kernel}), so every kernel runs in
    the cache and clock state it has in a real step.  Cold: every kernel of a layer again, round-robin over buffer
    sets whose footprints add up to more than three times the last-level cache, so nothing it reads is cached.
    Times in ms: {"mean", "median", "min"} per stage."""
    todo = [L for L in layers if not L.direct]
    plan = {id(L): stage_plan(torch, w, L, ws, 1) for L in todo}
    acc = {id(L): {name: [] for name, _ in plan[id(L)][0][0]} for L in todo}
    for rep in range(reps + 1):
        marks = []
        for L in layers:
            if L.direct:
                w.direct_conv2d_fwd(L.D, L.G, pad=1, Y=L.Y)
                continue
            for name, call in plan[id(L)][0][0]:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                call()
                e1.record()
                marks.append((id(L), name, e0, e1))
        torch.cuda.synchronize()
        if rep:
            for lid, name, e0, e1 in marks:
                acc[lid][name].append(e0.elapsed_time(e1))
    res = []
    for L in layers:
        if L.direct:
            res.append(None)
            continue
        _, nbytes, kernel, flops = plan[id(L)]
        st = {"variant": L.variant, "gemm_flops": flops, "bytes": nbytes, "kernel": kernel, "sets": 1}
        for name, ts in acc[id(L)].items():
            st[name] = stats(ts)
        res.append(st)
    del plan
    torch.cuda.empty_cache()
    if cold:
        for L, st in zip(layers, res):
            if st is None:
                continue
            foot = st["bytes"]["fused"] if "fused" in st["bytes"] else min(st["bytes"]["input"], st["bytes"]["output"])
            sets = n_sets(foot)
            plans, _, _, _ = stage_plan(torch, w, L, ws, sets)
            for j, (name, _) in enumerate(plans[0]):
                if name != "filter":
                    st[name + "_cold"] = time_calls(torch, [p[j][1] for p in plans], max(reps, sets))
            st["sets"] = sets
            del plans
            torch.cuda.empty_cache()
    return res


def summarize_stages(w, layers, stages, dtype, workload):
    """Per-layer rows, per-kernel totals, the roofline object of the dominant kernel and that of the transforms."""
    peak = PEAK["mfma_f32_TFs"] if dtype == "f32" else PEAK["mfma_f16_TFs"]
    rows, dom = [], {}
    hot = {"b": 0.0, "ms": 0.0}
    cold = {"b": 0.0, "ms": 0.0}
    per_kind = {}
    for L, st in zip(layers, stages):
        if st is None:
            continue
        main = "fused" if st["variant"] == w.FLAG_FUSED else "gemm"
        row = {"layer": L.name, "m": L.m, "variant": "fused" if main == "fused" else "unfused", "kernel": st["kernel"],
               "kernel_ms": st[main]["mean"], "kernel_ms_min": st[main]["min"],
               "kernel_tflops": st["gemm_flops"] / st[main]["mean"] / 1e9, "buffer_sets_cold": st["sets"]}
        if main + "_cold" in st:
            row["kernel_ms_cold"] = st[main + "_cold"]["median"]
        if main == "fused":
            # a one-kernel layer is bound by max(multiply flops / MFMA peak, (D + U + Y) / HBM peak)
            t_mfma, t_hbm = st["gemm_flops"] / (peak * 1e9), st["bytes"]["fused"] / (PEAK["hbm_GBs"] * 1e6)
            row["bound"] = "mfma" if t_mfma >= t_hbm else "hbm"
            row["bound_ms"] = max(t_mfma, t_hbm)
            row["frac_of_bound"] = max(t_mfma, t_hbm) / st[main]["mean"]
            row["GBs"] = st["bytes"]["fused"] / st[main]["mean"] / 1e6
        for k in ("filter", "input", "output"):
            if k in st:
                row[k + "_ms"] = st[k]["mean"]
                row[k + "_GBs"] = st["bytes"][k] / st[k]["mean"] / 1e6
                if k + "_cold" in st:
                    row[k + "_ms_cold"] = st[k + "_cold"]["median"]
                    row[k + "_GBs_cold"] = st["bytes"][k] / st[k + "_cold"]["median"] / 1e6
                if k != "filter":
                    hot["b"] += st["bytes"][k]
                    hot["ms"] += st[k]["mean"]
                    pk = per_kind.setdefault(k, {"b": 0.0, "hot": 0.0, "cold": 0.0})
                    pk["b"] += st["bytes"][k]
                    pk["hot"] += st[k]["mean"]
                    if k + "_cold" in st:
                        cold["b"] += st["bytes"][k]
                        cold["ms"] += st[k + "_cold"]["median"]
                        pk["cold"] += st[k + "_cold"]["median"]
        rows.append(row)
        d = dom.setdefault(st["kernel"], {"flops": 0.0, "ms": 0.0, "launches": 0, "bytes": 0.0, "min_ms": 0.0})
        d["flops"] += st["gemm_flops"]
        d["bytes"] += st["bytes"]["gemm"] if main == "gemm" else st["bytes"]["fused"]
        d["ms"] += st[main]["mean"]
        d["min_ms"] += st[main]["min"]
        d["launches"] += 1
    out = {"stages": rows}
    out["kernels"] = {k: {"launches_per_step": d["launches"], "avg_launch_ms": d["ms"] / d["launches"],
                          "tflops": d["flops"] / d["ms"] / 1e9, "frac_of_mfma_peak": d["flops"] / d["ms"] / 1e9 / peak,
                          "GBs": d["bytes"] / d["ms"] / 1e6, "frac_of_hbm_peak": d["bytes"] / d["ms"] / 1e6 / PEAK["hbm_GBs"]}
                      for k, d in dom.items()}
    if dom:
        # The dominant kernel is the kernel template with the largest share of the step; the library launches the
        # multiply in two block shapes (two instantiations of one template), which are one kernel here: its figures
        # are sums over all of its launches, the instances are listed with their launch counts and in `kernels`.
        fam = {}
        for k, v in dom.items():
            f = fam.setdefault(k.split("<")[0], {"flops": 0.0, "ms": 0.0, "launches": 0, "bytes": 0.0, "min_ms": 0.0,
                                                 "traffic": 0.0, "inst": []})
            for key in ("flops", "ms", "launches", "bytes", "min_ms"):
                f[key] += v[key]
            f["inst"].append((k, v["launches"]))
            t = MEASURED_TRAFFIC.get((workload, k))
            f["traffic"] = None if (t is None or f["traffic"] is None) else f["traffic"] + t * v["launches"]
        fname, d = max(fam.items(), key=lambda kv: kv[1]["ms"])
        name = d["inst"][0][0] if len(d["inst"]) == 1 else fname + ": " + " + ".join("%d x %s" % (n, k) for k, n in d["inst"])
        ach = d["flops"] / d["ms"] / 1e9
        roof = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                "traffic": None if d["traffic"] is None else d["traffic"] / d["launches"], "kernel": name,
                "launches_per_step": d["launches"], "avg_launch_ms": d["ms"] / d["launches"],
                "min_launch_ms": d["min_ms"] / d["launches"], "flops_per_launch": d["flops"] / d["launches"]}
        # a kernel whose flops per algorithmic byte fall below the machine balance (peak flops / peak bytes) is
        # bound by HBM, not by the matrix cores: the fp16-storage multiply (fp32 M written out) is
        if d["flops"] / d["bytes"] < peak * 1e12 / (PEAK["hbm_GBs"] * 1e9):
            gbs = d["bytes"] / d["ms"] / 1e6
            roof.update({"bound": "hbm", "achieved": gbs, "peak": PEAK["hbm_GBs"], "unit": "GB/s",
                         "frac": gbs / PEAK["hbm_GBs"], "bytes_per_launch": d["bytes"] / d["launches"],
                         "mfma_tflops": ach, "flops_per_byte": d["flops"] / d["bytes"]})
        out["roofline"] = roof
    if hot["ms"] > 0:
        use = cold if cold["ms"] > 0 else hot
        tr = {"bound": "hbm", "achieved": use["b"] / use["ms"] / 1e6, "peak": PEAK["hbm_GBs"], "unit": "GB/s",
              "frac": use["b"] / use["ms"] / 1e6 / PEAK["hbm_GBs"], "regime": "cold" if cold["ms"] > 0 else "hot",
              "hot_GBs": hot["b"] / hot["ms"] / 1e6,
              "kernels": "input_transform + output_transform of the four-stage layers"}
        for k, pk in per_kind.items():
            tr[k + "_GBs_hot"] = pk["b"] / pk["hot"] / 1e6
            if pk["cold"] > 0:
                tr[k + "_GBs_cold"] = pk["b"] / pk["cold"] / 1e6
        out["transform_roofline"] = tr
    return out


def stack_lower_bound(w, layers, dtype):
    """Launch-free lower bound of a step, layer by layer: max(multiply flops / MFMA peak, (D + U + Y) bytes / HBM
    peak) for a Winograd layer, (D + G + Y) bytes / HBM peak for the direct one; returns (ms, ms if only the
    multiplies counted, ms if only the bytes counted)."""
    peak = PEAK["mfma_f32_TFs"] if dtype == "f32" else PEAK["mfma_f16_TFs"]
    tot = mf = hb = 0.0
    for L in layers:
        s = L.D.element_size()
        if L.direct:
            b = (L.D.numel() + L.G.numel()) * s + L.Y.numel() * L.Y.element_size()
            t_m, t_h = 0.0, b / (PEAK["hbm_GBs"] * 1e6)
        else:
            a2 = (L.m + 2) ** 2
            b = L.D.numel() * s + a2 * L.K * L.C * s + L.Y.numel() * 4
            t_m, t_h = 2 * a2 * L.K * L.C * L.P / (peak * 1e9), b / (PEAK["hbm_GBs"] * 1e6)
        tot += max(t_m, t_h)
        mf += t_m
        hb += t_h
    return tot, mf, hb


def time_bwd_data(torch, w, layers, ws_bytes, steps):
    """Input gradient (Section 4.2 of the paper) of the 12 layers that need one (not the first):
    the error tensor is the layer's output buffer, same algorithm choice as the forward pass."""
    todo = [L for L in layers if not L.direct]
    if any(L.Y.dtype != L.D.dtype for L in todo):
        return None   # fp16 storage keeps fp32 outputs: no resident fp16 error tensor to time
    need = max(w.wino_workspace_bytes(L.N, L.K, L.HW, L.HW, L.C, 1, L.m, L.dt) for L in todo)
    ws = torch.empty(max(need, ws_bytes), dtype=torch.uint8, device="cuda")
    grads = [torch.empty_like(L.D, dtype=torch.float32) for L in todo]

    def step():
        for L, dD in zip(todo, grads):
            w.wino_conv2d_bwd_data(L.Y, G=L.G, pad=1, m=L.m, dD=dD, workspace=ws)
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
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        ev[0].record()
        for i in range(steps):
            w.wino_conv2d_bwd_filter(L.D, L.Y, pad=1, dG=dG, workspace=ws)
            ev[i + 1].record()
        torch.cuda.synchronize()
        sec = stats([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])["median"] / 1e3   # (a stray slow call is not the rate)
        per.append({"layer": L.name, "ms": sec * 1e3, "eff_tflops": L.flops / sec / 1e12})
    sec = sum(p["ms"] for p in per) / 1e3
    return {"eff_tflops": sum(L.flops for L in layers) / sec / 1e12, "ms_per_step": sec * 1e3, "layers": len(layers),
            "per_layer": per, "note": "effective flops as for the forward pass; per layer the median of the timed calls"}


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
           "layers_changed": [{"layer": L.name, "ms": t["mean"], "eff_tflops": L.flops / t["mean"] / 1e9}
                              for L, t in zip(changed, ms)]}
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


def time_graph(torch, w, layers, ws, steps, fx):
    """The whole step captured once in a HIP graph and replayed: removes the host's launch work, not the
    GPU's per-kernel start-up and drain.  Replays alternate with eager steps and are compared with them."""
    run_step(w, layers, ws, fx)
    torch.cuda.synchronize()
    refs = [L.Y.clone() for L in layers]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run_step(w, layers, ws, fx)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run_step(w, layers, ws, fx)
    torch.cuda.synchronize()
    same = True
    for _ in range(3):
        for L in layers:
            L.Y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        same = same and all(torch.equal(a, L.Y) for a, L in zip(refs, layers))
        run_step(w, layers, ws, fx)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return {"ms_per_step": (time.perf_counter() - t0) / steps * 1e3, "replays_equal_eager": bool(same)}


def cpu_baseline(torch, w, layers, budget_s=12.0, max_images=32):
    """The fp64 oracle (Eq. (1)) on the host cores over whole images of the same workload: image after image
    through all 13 layers until about `budget_s` seconds have been spent.  Its outputs are also the reference
    for the GPU outputs of those images (what the last step left in the layers' Y buffers)."""
    import numpy as np
    from oracle import direct
    flops, secs, imgs = 0.0, 0.0, 0
    nmax = layers[0].N
    worst = {}
    while secs < budget_s and imgs < min(max_images, nmax):
        for L in layers:
            D = L.D_host[imgs:imgs + 1]
            t0 = time.perf_counter()
            ref = direct.conv2d_fwd(D, L.G_host, pad=1)
            secs += time.perf_counter() - t0
            flops += direct_flops(1, L.C, L.HW, L.HW, L.K)
            got = L.Y[imgs:imgs + 1].float().cpu().numpy().astype(np.float64)
            e = float(np.linalg.norm((got - ref).ravel()) / np.linalg.norm(ref.ravel()))
            worst[L.name] = max(worst.get(L.name, 0.0), e)
        imgs += 1
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": direct.num_threads(), "kind": "oracle",
            "images_per_sec": imgs / secs,
            "sample": "fp64 direct convolution of all 13 layers, %d image(s) of the batch of %d, %.1f s of CPU time"
                      % (imgs, nmax, secs),
            "gpu_vs_oracle_rel_err": {"max": max(worst.values()), "per_layer": worst,
                                      "note": "normwise relative error of the GPU outputs of the sampled images"}}


def algorithm_text(policy):
    if policy == "auto":
        return "F(4x4,3x3) where 4 divides H, else F(2x2,3x3); conv1.1 direct"
    if policy == "auto_n1":
        return "F(4x4,3x3) for images of 56x56 and more, else F(2x2,3x3); conv1.1 direct"
    return "F(%sx%s,3x3); conv1.1 direct" % (policy, policy)


def stack_leg(torch, w, args, N, dtype, policy, cfg_idx, steps, warmup, cold=True, baseline=False):
    """One VGG-16 stack workload, measured in full; returns the dictionary of its figures."""
    import numpy as np
    from paper_1509_09308_amd import synth
    np_dtype = np.float32 if dtype == "f32" else np.float16
    layers = make_layers(N, np_dtype, policy, cfg_idx)
    ws = torch.empty(max(L.ws_bytes for L in layers if not L.direct), dtype=torch.uint8, device="cuda")
    total_flops = sum(L.flops for L in layers)
    workload = "vgg16_3x3_conv_stack_N%d_%s" % (N, dtype)

    sec = time_steps(torch, w, layers, ws, steps, warmup)
    out = {"value": total_flops / sec / 1e12, "unit": "TFLOP/s", "ms_per_step": sec * 1e3, "steps": steps, "warmup": warmup,
           "dtype": dtype,
           "config": {"workload": workload, "batch": N, "layers": 13, "algorithm": algorithm_text(policy),
                      "filter_transform": "inside the timed step"},
           "images_per_sec": N / sec, "direct_gflop_per_step": total_flops / 1e9}
    out["step_ms"] = time_steps_events(torch, w, layers, ws, max(steps, 10))
    layer_ms = time_layers(torch, w, layers, ws, max(5, steps))
    out["per_layer"] = [{"layer": L.name, "m": L.m, "ms": t["mean"], "ms_median": t["median"], "ms_min": t["min"],
                         "eff_tflops": L.flops / t["mean"] / 1e9} for L, t in zip(layers, layer_ms)]
    # the same per-layer times re-weighted with the depths of VGG network E (Table 3 of the paper)
    shape = lambda L: (L.C, L.HW, L.K)
    count16 = {}
    for L in layers:
        count16[shape(L)] = count16.get(shape(L), 0) + 1
    wE = [synth.VGG_E_DEPTH[shape(L)] / count16[shape(L)] for L in layers]
    e_flops = sum(x * L.flops for x, L in zip(wE, layers))
    e_ms = sum(x * t["mean"] for x, t in zip(wE, layer_ms))
    out["vgg_e_weighted"] = {"eff_tflops": e_flops / e_ms / 1e9, "ms": e_ms,
                             "paper_titanx_f2x2_tflops": PAPER_TITANX["fp32" if dtype == "f32" else "fp16"].get(N)}
    lb, lb_m, lb_h = stack_lower_bound(w, layers, dtype)
    out["lower_bound"] = {"ms": lb, "mfma_only_ms": lb_m, "hbm_only_ms": lb_h, "frac": lb / (sec * 1e3),
                          "note": "sum over layers of max(multiply flops / MFMA peak, (D + U + Y) bytes / HBM peak)"}

    # FX (Section 6): filters transformed once, ahead of the step
    for L in layers:
        if not L.direct:
            L.U = w.wino_filter_transform(L.G, L.m)
    torch.cuda.synchronize()
    fsec = time_steps(torch, w, layers, ws, steps, warmup, fx=True)
    out["fx"] = {"ms_per_step": fsec * 1e3, "eff_tflops": total_flops / fsec / 1e12, "images_per_sec": N / fsec,
                 "note": "filters pre-transformed by wino_filter_transform outside the timed region"}

    if dtype == "f16":
        # the same step with fp16 outputs (the workload's definition keeps Y in fp32; this is the other reading)
        keep = [L.Y for L in layers]
        for L in layers:
            L.Y = torch.empty_like(L.Y, dtype=torch.float16)
        ysec = time_steps(torch, w, layers, ws, steps, warmup)
        out["fp16_outputs"] = {"ms_per_step": ysec * 1e3, "eff_tflops": total_flops / ysec / 1e12,
                               "note": "Y stored in fp16 instead of fp32 (one rounding more; not the headline of this leg)"}
        for L, y in zip(layers, keep):
            L.Y = y
    if not args.no_stages:
        stages = time_stages(torch, w, layers, ws, max(5, steps), cold=cold)
        out.update(summarize_stages(w, layers, stages, dtype, workload))
        if "transform_roofline" not in out:
            # The step runs every Winograd layer in one kernel: the four stages of Algorithm 1 as kernels of their own
            # are measured beside it, on the last layer of each algorithm forced through them.
            import copy
            ref_layers = []
            for m in sorted({L.m for L in layers if not L.direct}):
                L = copy.copy([x for x in layers if not x.direct and x.m == m][-1])
                L.variant = w.FLAG_UNFUSED
                ref_layers.append(L)
            ref = summarize_stages(w, ref_layers, time_stages(torch, w, ref_layers, ws, max(5, steps), cold=cold), dtype, workload)
            out["four_stage_reference"] = {"layers": [L.name for L in ref_layers], "stages": ref["stages"], "kernels": ref["kernels"],
                                           "note": "not part of the step: these layers forced through the four stages"}
            if "transform_roofline" in ref:
                tr = dict(ref["transform_roofline"])
                tr["kernels"] = "input_transform + output_transform of %s forced through the four stages (the step runs none)" \
                                % " and ".join("%s (m=%d)" % (L.name, L.m) for L in ref_layers)
                out["transform_roofline"] = tr
    if baseline and not args.no_cpu_baseline:
        run_step(w, layers, ws)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(torch, w, layers)
    return out, layers, ws, [t["mean"] for t in layer_ms]


def n1_leg(torch, w, args, dtype, policy):
    steps, warmup = max(args.steps, 20), max(args.warmup, 5)
    out, layers, ws, _ = stack_leg(torch, w, args, 1, dtype, policy, 3, steps, warmup, cold=False)
    out["algorithm"] = {L.name: ("direct" if L.direct else "F(%dx%d,3x3)" % (L.m, L.m)) for L in layers}
    out["eff_tflops"] = out["value"]
    # bound of the step: what it would take with no launch cost at all
    lb = out["lower_bound"]
    flops = sum(2 * (L.m + 2) ** 2 * L.K * L.C * L.P for L in layers if not L.direct)
    peak = PEAK["mfma_f32_TFs"] if dtype == "f32" else PEAK["mfma_f16_TFs"]
    ach = flops / out["ms_per_step"] / 1e9
    out["roofline"] = {"bound": "mfma" if lb["mfma_only_ms"] >= lb["hbm_only_ms"] else "hbm", "achieved": ach, "peak": peak,
                       "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
                       "kernel": "whole step (all launches)", "frac_of_launch_free_bound": lb["frac"],
                       "launch_free_bound_ms": lb["ms"]}
    out["hip_graph"] = time_graph(torch, w, layers, ws, steps, fx=False)
    out["hip_graph_fx"] = time_graph(torch, w, layers, ws, steps, fx=True)
    if dtype == "f32":
        out["one_launch_per_layer"] = time_one_launch(torch, w, layers, steps, warmup)
    return out


def single_layer_leg(torch, w, args, N, C, HW, K, ms_list, cfg_idx, name):
    """A one-layer workload through wino_conv2d_fwd_ex for every m in ms_list, with its stage times."""
    import numpy as np
    out = {"config": {"workload": name, "N": N, "C": C, "K": K, "H": HW, "W": HW, "dtype": "f32"}}
    for m in ms_list:
        layers = make_layers(N, np.float32, str(m), cfg_idx, shapes=[("layer", C, HW, K)])
        L = layers[0]
        ws = torch.empty(L.ws_bytes, dtype=torch.uint8, device="cuda")
        steps, warmup = max(args.steps, 20), max(args.warmup, 5)
        sec = time_steps(torch, w, layers, ws, steps, warmup)
        r = {"ms": sec * 1e3, "eff_tflops": L.flops / sec / 1e12, "step_ms": time_steps_events(torch, w, layers, ws, steps)}
        if not args.no_stages:
            st = time_stages(torch, w, layers, ws, 10, cold=True)
            sm = summarize_stages(w, layers, st, "f32", name)
            r["stages"] = sm["stages"][0]
            r["roofline"] = sm.get("roofline")
        out["F(%dx%d,3x3)" % (m, m)] = r
    return out


def probe(torch, w, layers, ws):
    """For rocprofv3 --pmc runs: one 1 GiB device copy (counter calibration), then every kernel of one step
    twice (hot); prints the algorithmic bytes per kernel."""
    a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    b.copy_(a)                                                      # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del a, b
    st = time_stages(torch, w, layers, ws, 1, cold=False)
    print(json.dumps({"probe": "1 GiB copy, then each kernel of one step twice (warm-up + timed)",
                      "layers": [{"layer": L.name, "kernel": x["kernel"], "flops": x["gemm_flops"],
                                  "bytes": x["bytes"]} for L, x in zip(layers, st) if x]}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--dtype", choices=["f32", "f16"], default="f32")
    ap.add_argument("--m", default="auto", help="auto | 2 | 4 | 6 (6: fp32 only)")
    ap.add_argument("--only", choices=LEGS, default=None,
                    help="run one leg only (headline = the N=64 fp32 stack with --batch/--dtype/--m applied)")
    ap.add_argument("--no-n1", action="store_true")
    ap.add_argument("--no-f16", action="store_true", help="skip the fp16-storage N=32 leg")
    ap.add_argument("--no-single", action="store_true", help="skip the two single-layer workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stages", action="store_true")
    ap.add_argument("--no-bwd", action="store_true", help="skip the input- and filter-gradient lines")
    ap.add_argument("--no-f6", action="store_true", help="skip the F(6x6,3x3) and all-F(4x4,3x3) lines")
    ap.add_argument("--steps-only", action="store_true",
                    help="for rocprofv3 --kernel-trace --stats: warm-up and timed steps of the chosen leg, nothing else")
    ap.add_argument("--grads", action="store_true",
                    help="with --steps-only: the input- and filter-gradient steps of the leg instead of forward steps")
    ap.add_argument("--probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (counter calibration), then every "
                         "kernel of one step of the chosen leg twice; prints the algorithmic bytes per kernel and exits")
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
    only = args.only
    if only == "f16":
        args.batch, args.dtype = 32, "f16"
    elif only == "n1":
        args.batch, args.dtype = 1, "f32"
    cfg_idx = {("f32", 1): 3, ("f16", 1): 3}.get((args.dtype, args.batch), 4 if args.dtype == "f32" else 5)
    policy = args.m if args.dtype == "f32" else ("4" if args.m == "auto" else args.m)
    if args.batch == 1 and args.dtype == "f32" and policy == "auto":
        policy = "auto_n1"

    if args.probe or args.steps_only:
        if only == "cfg2" or only == "cfg1":
            shp = [("layer", 512, 28, 512)] if only == "cfg2" else [("layer", 32, 56, 32)]
            layers = make_layers(8 if only == "cfg2" else 1, np.float32, "4" if (only == "cfg2" and args.m == "auto") else
                                 ("2" if args.m == "auto" else args.m), 2 if only == "cfg2" else 1, shapes=shp)
        else:
            layers = make_layers(args.batch, np.float32 if args.dtype == "f32" else np.float16, policy, cfg_idx)
        ws = torch.empty(max(L.ws_bytes for L in layers if not L.direct), dtype=torch.uint8, device="cuda")
        if args.probe:
            probe(torch, w, layers, ws)
        elif args.grads:
            run_step(w, layers, ws)   # the error tensors of the gradient steps are the forward outputs
            bd = time_bwd_data(torch, w, layers, ws.numel(), args.steps)
            bf = time_bwd_filter(torch, w, layers, args.steps)
            print(json.dumps({"steps_only": True, "grads": True, "bwd_data": bd, "bwd_filter": bf}))
        else:
            sec = time_steps(torch, w, layers, ws, args.steps, args.warmup)
            print(json.dumps({"steps_only": True, "ms_per_step": sec * 1e3, "steps": args.steps, "warmup": args.warmup,
                              "launch_rounds": args.steps + args.warmup}))
        return

    lib_hash = w.build.built_hash()
    if only in ("cfg2", "cfg1"):
        leg = single_layer_leg(torch, w, args, 8, 512, 28, 512, (2, 4), 2, "vgg_layer_512_512_28x28_N8_f32") if only == "cfg2" \
            else single_layer_leg(torch, w, args, 1, 32, 56, 32, (2,), 1, "layer_32_32_56x56_N1_f32")
        leg["lib_hash"] = lib_hash
        print(json.dumps(leg))
        return
    if only == "n1":
        leg = n1_leg(torch, w, args, args.dtype, policy)
        leg["lib_hash"] = lib_hash
        print(json.dumps(leg))
        return

    head, layers, ws, layer_ms = stack_leg(torch, w, args, args.batch, args.dtype, policy, cfg_idx, args.steps, args.warmup,
                                           cold=True, baseline=True)
    out = {"metric": "effective conv TFLOPS, VGG-16 3x3 conv stack forward, N=%d, 1 GPU" % args.batch,
           "value": head.pop("value"), "unit": head.pop("unit"), "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": args.dtype, "data": "synthetic", "config": head.pop("config"), "lib_hash": lib_hash}
    for k in ("steps", "warmup", "dtype"):
        head.pop(k, None)
    out.update(head)

    main_leg = only is None or only == "headline"
    if main_leg and not args.no_bwd:
        bd = time_bwd_data(torch, w, layers, ws.numel(), max(3, args.steps // 2))
        if bd:
            out["bwd_data"] = bd
        bf = time_bwd_filter(torch, w, layers, max(3, args.steps // 2))
        if bf:
            out["bwd_filter"] = bf
    if main_leg and not args.no_f6 and policy == "auto" and args.dtype == "f32":
        f4 = time_all_f4x4(torch, w, layers, args.steps, args.warmup)
        if f4:
            out["all_f4x4"] = f4
        f6 = time_f6x6(torch, w, layers, layer_ms, max(3, args.steps // 2))
        if f6:
            out["f6x6"] = f6
    del layers, ws
    torch.cuda.empty_cache()
    if only is None and args.batch == 64 and args.dtype == "f32":
        if not args.no_f16:
            leg, l5, ws5, _ = stack_leg(torch, w, args, 32, "f16", "4", 5, args.steps, args.warmup, cold=True)
            out["cfg5_f16_n32"] = leg
            del l5, ws5
            torch.cuda.empty_cache()
        if not args.no_n1:
            out["n1"] = n1_leg(torch, w, args, "f32", "auto_n1" if policy == "auto" else policy)
            torch.cuda.empty_cache()
        if not args.no_single:
            out["cfg2"] = single_layer_leg(torch, w, args, 8, 512, 28, 512, (2, 4), 2, "vgg_layer_512_512_28x28_N8_f32")
            out["cfg1"] = single_layer_leg(torch, w, args, 1, 32, 56, 32, (2,), 1, "layer_32_32_56x56_N1_f32")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
