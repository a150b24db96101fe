#!/usr/bin/env python3
"""Benchmark of the splatting hot path on one MI355X.

A step = one pass of the whole per-view path over one synthetic view, inputs resident in HBM:
    pbdr_preprocess -> pbdr_render_fwd -> pbdr_render_bwd (which, as the first view of its batch, also zeroes the
    parameter-gradient entries of points the view does not use; --separate-zero does that with a fill of its own)
on the 1M-Gaussian / SH degree 3 / 1920x1080 configuration (fwd+bwd views per second).  dL/dimage is the gradient of
a mean-L1 loss against a seeded target, computed once from the warm-up image (the loss itself is harness, not path).

Prints ONE JSON line with the contract fields plus
  `roofline`       dominant kernel, timed live with HIP events recorded on the launch stream inside the timed region;
                   flop fraction of the fp32 vector peak and, from the committed shader-counter profile, the share of
                   the vector ALU's issue capacity its instructions take (`valu_issue_frac`);
  `cpu_baseline`   the CPU oracle timed on the host cores on one full view;
  `step_ms`        median / min / max of single steps (one event pair per step, after the timed region);
  `measured_peaks` plain-FMA rate of this machine (a child process run before the GPU is touched) and a device copy;
  `configs`        the other benchmark configurations, each a short timed loop of its own: the tiny scene, the batch of 16
                   views, the 8M-point street scene as a batch of 8 views at 4K with point-group culling, 2D surfels -
                   with throughput, dominant kernel, pairs / cull rate, staged parity and the oracle's time on one view.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published MI355X peaks
HBM_PEAK_GBS = 8000.0
# fp32 vector: the published 157.3 TFLOP/s = 256 CUs x 4 SIMDs x 32 lanes x 2 flop x 2.4 GHz. The library is built with
# packed fp32 disabled, but plain v_fma_f32 does not run at half of that: a micro-benchmark of independent plain FMAs
# reaches 116.6 TFLOP/s on this part (2.7 cycles per wave64 instruction per SIMD), so the published figure is the peak.
ALU_PEAK_TFLOPS = 256 * 4 * 32 * 2 * 2.4e9 / 1e12

# algorithmic work per unit: flops per examined and per blended (pixel, splat) pair
FWD_FLOPS_PER_EXAMINED = 12.0    # 2 sub, 8 for the quadratic form, exp, opacity mul (+ min / compares not counted)
FWD_FLOPS_PER_BLENDED = 9.0      # 1-alpha, T', w, 3 fma
BWD_FLOPS_PER_EXAMINED = 12.0    # alpha recomputed
BWD_FLOPS_PER_BLENDED = 53.0     # 44 for the per-pair gradient terms + 9 lane-sum adds
# surfels: 2 sub, 12 for h_u and h_v, 9 for the cross product, reciprocal, 2 for (u, v), 4 + 3 for the two exponents,
# max, opacity add, exp2
FWD2D_FLOPS_PER_EXAMINED = 36.0
BWD2D_FLOPS_PER_BLENDED = 55.0   # 40 for the per-pair gradient terms and moments + 15 lane-sum adds


def profiled_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE in KiB,
    scaled by what the same counters read for a plain copy of known size); None if the summary does not cover it."""
    path = os.path.join(ROOT, "profiles", "bench_mid_pmc_traffic.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    scale_f = scale_w = None
    for ln in lines:
        if ln.startswith("scale_fetch="):
            parts = dict(kv.split("=") for kv in ln.split())
            scale_f, scale_w = float(parts["scale_fetch"]), float(parts["scale_write"])
    if scale_f is None:
        return None
    for ln in lines:
        cols = ln.split("\t")
        if len(cols) == 3 and cols[0].split("::")[-1].split("<")[0] == kernel:
            return (float(cols[1]) * scale_f + float(cols[2]) * scale_w) * 1024.0
    return None


def profiled_valu_cycles(kernel):
    """Vector-ALU issue cycles per launch of `kernel`, summed over the chip's SIMDs, from the committed shader-counter
    summary of the benchmark workload: SQ_INSTS_VALU wavefront instructions at the cost of a plain instruction plus the
    extra cost of the transcendental ones (SQ_INSTS_VALU_TRANS_F32), both costs calibrated on the FMA / exp micro-benchmark
    (profiles/valu_issue_pmc_calibration.txt: a kernel of plain FMAs that keeps every SIMD issuing reads one SQ_INSTS_VALU
    per instruction). DPP and row-swap instructions cost more than a plain one too and have no counter of their own, so
    this is a lower bound of the kernel's share of the issue capacity. None if a file or the kernel is missing."""
    try:
        cal = open(os.path.join(ROOT, "profiles", "valu_issue_pmc_calibration.txt")).read().splitlines()
        rows = open(os.path.join(ROOT, "profiles", "bench_mid_pmc_sq.txt")).read().splitlines()
    except OSError:
        return None
    c_plain = c_trans = None
    for ln in cal:
        if ln.startswith("cycles_per_plain_inst="):
            parts = dict(kv.split("=") for kv in ln.split())
            c_plain, c_trans = float(parts["cycles_per_plain_inst"]), float(parts["cycles_per_trans_inst"])
    header = None
    for ln in rows:
        cols = ln.split("\t")
        if cols[0] == "kernel":
            header = cols
        elif header and len(cols) == len(header) and cols[0].split("::")[-1].split("<")[0] == kernel and c_plain:
            rec = dict(zip(header, cols))
            return float(rec["SQ_INSTS_VALU"]) * c_plain + float(rec["SQ_INSTS_VALU_TRANS_F32"]) * (c_trans - c_plain)
    return None


def measured_peaks():
    """The instruction-issue micro-benchmark as a child process, before this process touches the GPU: the rate of
    independent plain v_fma_f32 this box reaches (the fp32 vector peak reachable without packed math)."""
    import re
    import subprocess
    exe = os.path.join(ROOT, "paper_2512_20017_amd", "ubench", "valu_issue.bin")
    if not os.path.exists(exe):
        try:
            from paper_2512_20017_amd import build as hip_build
            hip_build.build_ubench()
        except Exception:
            return None
    try:
        txt = subprocess.run([exe], capture_output=True, text=True, timeout=120).stdout
    except Exception:
        return None
    m = re.search(r"plain v_fma_f32[^:]*: ([0-9.]+) TFLOP/s, ([0-9.]+) cycles", txt)
    if not m:
        return None
    out = dict(fma_tflops=float(m.group(1)), cycles_per_plain_inst=float(m.group(2)))
    for key, pat in (("cycles_per_dpp_add", r"v_add_f32_dpp\s+([0-9.]+)"), ("cycles_per_exp", r"v_exp_f32\s+([0-9.]+)"),
                     ("cycles_per_row_swap", r"v_permlane16_swap_b32\s+([0-9.]+)")):
        mm = re.search(pat, txt)
        if mm:
            out[key] = float(mm.group(1))
    return out


def per_step_times(torch, step, count):
    """One event pair per step on the current stream; returns the steps' durations in ms."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)]
    torch.cuda.synchronize()
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in ev]


def spread(ms_list):
    xs = sorted(ms_list)
    return dict(median_ms=xs[len(xs) // 2], min_ms=xs[0], max_ms=xs[-1], steps=len(xs))


def oracle_view_check(np, oracle, sc, cam, sp_np, image_chw, P_gpu, bg, dL_chw, surfels=False, time_full=True):
    """The CPU oracle on one view: (1) timed from raw parameters through forward and backward on the host cores; (2) its
    compositing fed with the GPU's own fp32 splat state, for the staged parity figures over the whole image."""
    import time as _t
    W, H = cam["width"], cam["height"]
    keys = ("mean2d", "T", "opacity", "color") if surfels else ("mean2d", "conic", "opacity", "color")
    o_pre, o_fwd, o_bwd, o_pbwd = ((oracle.preprocess2d, oracle.render_fwd2d, oracle.render_bwd2d, oracle.preprocess_bwd2d)
                                   if surfels else
                                   (oracle.preprocess, oracle.render_fwd, oracle.render_bwd, oracle.preprocess_bwd))
    cpu = None
    if time_full:
        t0 = _t.perf_counter()
        o_sp = o_pre(sc, cam)
        st = {k: o_sp[k].astype(np.float32).astype(np.float64) for k in keys}
        st["radius"] = o_sp["radius"]
        lists = oracle.bin_sort(st["mean2d"], st["radius"], o_sp["depth"].astype(np.float32), W, H)
        o_fwd(st, lists, W, H, bg)
        G = dL_chw.permute(1, 2, 0).contiguous().cpu().numpy().astype(np.float64)
        o_b = o_bwd(st, lists, W, H, bg, G)
        o_pbwd(sc, cam, o_b)
        t1 = _t.perf_counter()
        cpu = dict(value=1.0 / (t1 - t0), unit="views/s", cores=oracle.num_threads(), kind="oracle",
                   sample="1 full view (forward + backward) of the same workload, fp64, OpenMP", seconds=t1 - t0)
    stg = {k: sp_np[k].astype(np.float64) for k in keys}
    stg["radius"] = sp_np["radius"]
    lg = oracle.bin_sort(stg["mean2d"], stg["radius"], sp_np["depth"], W, H)
    rf = o_fwd(stg, lg, W, H, bg)
    got = image_chw.permute(1, 2, 0).cpu().numpy()
    ok = rf["fragile"] == 0
    parity = dict(max_abs_image_err=float(np.abs(got - rf["image"])[ok].max()), fragile_pixels=int((~ok).sum()),
                  pairs_oracle=int(lg["P"]), pairs_gpu=int(P_gpu), examined_oracle=int(rf["n_eval"]),
                  blended_oracle=int(rf["n_blend"]))
    return cpu, parity, rf


def bench_batch(args, workload, nb, group, streams, steps, with_oracle=True):
    """The B views of a batch (Alg. 1 lines 2-4 and 21-24 for a batch): preprocessing and its backward for the whole batch in
    one pass over the points each (pbdr_preprocess_batch, pbdr_preprocess_bwd_batch, optionally with point-group culling),
    the views rendered between them on `streams` streams; next to the same work with the per-view calls. One step = one
    batch; views_per_s counts views. workload: "mid" (1M points, 16 cameras on a sphere, 1080p) or "large" (8M points,
    8 street-level cameras at 4K)."""
    import numpy as np
    import torch

    from paper_2512_20017_amd import binding as B
    from paper_2512_20017_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()
    if workload == "large":
        sc = synth.scene_large(args.seed)
        cams = synth.cameras_street(args.seed)[:nb]
        wl = f"large, batched: 8M Gaussians, SH degree 3, street-level cameras 0..{nb - 1} of 8 at 3840x2160"
    else:
        sc = synth.scene_mid(args.seed)
        cams = synth.cameras_sphere()[:nb]
        wl = f"batched: the mid scene (1M Gaussians, SH degree 3) from cameras 0..{nb - 1} of 16, 1920x1080"
    nb = len(cams)
    n = int(sc["mean"].shape[0])
    W, H = cams[0]["width"], cams[0]["height"]
    bg = [0.0, 0.0, 0.0]
    scene = B.Scene.from_numpy(sc)
    splats = [B.Splats.empty(n) for _ in cams]
    g_splats = [B.SplatGrads.empty(n) for _ in cams]
    grads = scene.zeros_like()
    image = torch.empty((3, H, W), device="cuda")
    final_T = torch.empty((H, W), device="cuda")
    last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")
    bounds = keep = None
    if group > 0:
        ng = B.pbdr_group_count(n, group)
        bounds = torch.empty((7, ng), dtype=torch.float32, device="cuda")
        keep = torch.empty((nb, ng), dtype=torch.uint8, device="cuda")
        keep1 = torch.empty(ng, dtype=torch.uint8, device="cuda")
        B.pbdr_group_bounds(scene, group, bounds)
    # pair capacity: the largest view's count
    cap = max(min(16 * n, 32_000_000), 1 << 16)
    ws = B.alloc_workspace(n, W, H, cap)
    B.pbdr_preprocess_batch(scene, cams, splats, group, bounds, keep)
    pairs, visible = [], []
    for v, cam in enumerate(cams):
        B.pbdr_render_fwd(splats[v], cam, bg, cap, image, final_T, last_idx, ws)
        P, over = B.pbdr_query_lists(ws, n, W, H, cap)
        assert not over
        pairs.append(int(P))
        visible.append(int((splats[v].radius > 0).sum().item()))
    del ws
    cap = int(max(pairs) * 1.25) + 4096
    ws = B.alloc_workspace(n, W, H, cap)
    dL = torch.full((3, H, W), 1.0 / float(3 * W * H), device="cuda")
    dL[:, ::2, 1::2] *= -1.0

    # the views of a batch are independent between the two batched calls: they are rendered on `ns` streams, each with
    # its own workspace and outputs
    ns = max(1, min(streams, nb))
    main = torch.cuda.current_stream()
    lanes = [dict(stream=torch.cuda.Stream(), ws=B.alloc_workspace(n, W, H, cap), image=torch.empty((3, H, W), device="cuda"),
                  final_T=torch.empty((H, W), device="cuda"), last_idx=torch.empty((H, W), dtype=torch.int32, device="cuda"))
             for _ in range(ns)] if ns > 1 else []

    def step_batch():
        B.pbdr_preprocess_batch(scene, cams, splats, group, bounds, keep)
        if ns == 1:
            for v, cam in enumerate(cams):
                B.pbdr_render_fwd(splats[v], cam, bg, cap, image, final_T, last_idx, ws)
                B.pbdr_render_bwd(None, splats[v], cam, bg, cap, final_T, last_idx, dL, g_splats[v], None, ws)
        else:
            ready = torch.cuda.Event()
            ready.record(main)
            for k, ln in enumerate(lanes):
                ln["stream"].wait_event(ready)
                with torch.cuda.stream(ln["stream"]):
                    for v in range(k, nb, ns):
                        B.pbdr_render_fwd(splats[v], cams[v], bg, cap, ln["image"], ln["final_T"], ln["last_idx"], ln["ws"])
                        B.pbdr_render_bwd(None, splats[v], cams[v], bg, cap, ln["final_T"], ln["last_idx"], dL, g_splats[v], None,
                                          ln["ws"])
                done = torch.cuda.Event()
                done.record(ln["stream"])
                main.wait_event(done)
        B.pbdr_preprocess_bwd_batch(scene, cams, splats, g_splats, grads, first_view=True)

    def step_per_view():
        for v, cam in enumerate(cams):
            if group > 0:
                B.pbdr_preprocess_grouped(scene, cam, group, bounds, keep1, splats[v])
            else:
                B.pbdr_preprocess(scene, cam, splats[v])
            B.pbdr_render_fwd(splats[v], cam, bg, cap, image, final_T, last_idx, ws)
            B.pbdr_render_bwd(scene, splats[v], cam, bg, cap, final_T, last_idx, dL, None, grads, ws, first_view=(v == 0))

    names = B.profile_kernel_names()
    out = {}
    for label, step in (("batch_calls", step_batch), ("per_view_calls", step_per_view)):
        for _ in range(max(args.warmup, 1) if label == "batch_calls" else 1):
            step()
        torch.cuda.synchronize()
        B.pbdr_profile_begin((1 << len(names)) - 1, 64 * nb * 2)
        step()
        torch.cuda.synchronize()
        kern = {}
        for kid, name in enumerate(names):
            ms, cnt = B.pbdr_profile_collect(kid)
            if cnt:
                kern[name] = dict(ms_per_batch=ms, launches=cnt)
        B.pbdr_profile_end()
        torch.cuda.synchronize()
        k_steps = steps if label == "batch_calls" else max(2, steps // 3)
        t0 = time.perf_counter()
        for _ in range(k_steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        out[label] = dict(views_per_s=nb * k_steps / (t1 - t0), ms_per_batch=(t1 - t0) * 1e3 / k_steps, steps=k_steps,
                          kernels={k: kern[k] for k in ("k_preprocess", "k_preprocess_bwd", "k_group_cull", "k_composite_fwd",
                                                        "k_composite_bwd") if k in kern})
        if label == "batch_calls":
            out[label].update(spread(per_step_times(torch, step, max(5, min(20, steps)))))
    res = {
        "metric": "fwd+bwd views/sec, batch of views (not the headline)",
        "value": out["batch_calls"]["views_per_s"], "unit": "views/s", "ms_per_view": out["batch_calls"]["ms_per_batch"] / nb,
        "config": {"workload": wl, "n_gaussians": n, "width": W, "height": H, "views_per_batch": nb, "group_size": group,
                   "render_streams": ns, "pairs_per_view": pairs, "visible_per_view": visible,
                   "cull_rate": 1.0 - float(sum(visible)) / float(nb * n),
                   "groups_kept": float(keep.float().mean().item()) if group > 0 else None},
        "batch_calls": out["batch_calls"], "per_view_calls": out["per_view_calls"]}
    if with_oracle:
        import oracle
        # the view with the most pairs, alone: the oracle timed on it, and the staged parity of its image
        v = int(np.argmax(pairs))
        B.pbdr_render_fwd(splats[v], cams[v], bg, cap, image, final_T, last_idx, ws)
        torch.cuda.synchronize()
        cpu, parity, _ = oracle_view_check(np, oracle, sc, cams[v], splats[v].to_numpy(), image, pairs[v], bg, dL)
        res["cpu_baseline"] = cpu
        res["parity"] = dict(parity, view=v)
    return res


def run_batched(args):
    res = bench_batch(args, args.workload if args.workload in ("mid", "large") else "mid", args.batch_views, args.group_size,
                      args.streams, args.steps, with_oracle=not args.no_cpu_baseline)
    res.update({"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["batch_calls"]["ms_per_batch"],
                "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"})
    print(json.dumps(res))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mid", choices=["mid", "tiny", "surfels", "large"],
                    help="mid = the headline configuration; surfels = the same with 2D Gaussian disks (not the headline metric)")
    ap.add_argument("--group-size", type=int, default=0,
                    help="if > 0: preprocess with point-group frustum culling at this group size (3D Gaussian workloads)")
    ap.add_argument("--batch-views", type=int, default=0,
                    help="if > 0: time a batch of this many views (at most 16) of the mid scene with the batched "
                         "preprocessing calls, next to the per-view calls; not the headline metric")
    ap.add_argument("--train-step", action="store_true",
                    help="time a whole training iteration instead (Alg. 1 on one GPU: splat, render, L1 loss, backward, "
                         "selective Adam; with --separate-zero the Adam pass also zeroes the consumed gradient entries and the "
                         "backward accumulates); not the headline metric")
    ap.add_argument("--unfused-adam", action="store_true",
                    help="with --train-step: splatting backward into the gradient buffer, then pbdr_adam_selective per "
                         "attribute, instead of the one-pass pbdr_preprocess_bwd_batch_adam")
    ap.add_argument("--separate-zero", action="store_true",
                    help="clear the gradient buffer with a separate fill each step and accumulate into it, instead of "
                         "letting the backward call write it as the first view of its batch")
    ap.add_argument("--streams", type=int, default=3,
                    help="after the timed region, also time the same step with this many views in flight on separate "
                         "streams (reported as `overlapped`, not as `value`); 1 = skip. With --batch-views: the streams "
                         "the views of a batch are rendered on")
    ap.add_argument("--splat-grads", action="store_true",
                    help="have pbdr_render_bwd also write dL/d(splat state) out (nine planes), which the step itself does not need")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the leg that replays the step from a HIP graph")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-secondary", action="store_true", help="skip the other configurations after the headline")
    ap.add_argument("--no-peaks", action="store_true", help="skip the child process that measures the FMA issue rate")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (a kernel of known traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.batch_views > 0:
        assert args.batch_views <= 16 and args.workload in ("mid", "large")
        if args.steps == 50:
            args.steps = 10
        run_batched(args)
        return

    # the micro-benchmark of the vector ALU's issue rate, as a child process, before this process touches the GPU
    peaks = None if args.no_peaks else measured_peaks()
    out = bench_view(args, args.workload, headline=True)
    out["measured_peaks"] = dict(peaks or {}, device_copy_gbs=out.get("device_copy_gbs"))
    if peaks and out["roofline"].get("bound") == "alu":
        out["roofline"]["frac_of_measured_fma"] = out["roofline"]["achieved"] / peaks["fma_tflops"]
    if args.workload == "mid" and not args.train_step and not args.no_secondary:
        out["configs"] = secondary_configs(args)
    print(json.dumps(out))


def secondary_configs(args):
    """The other benchmark configurations, each a short timed loop after the headline's timed region (their figures are
    not `value`): the tiny scene, the batch of 16 views of the 1M scene, the 8 street-level 4K views of the 8M scene as a
    batch with point-group culling, and the 2D surfel variant."""
    import copy
    import gc

    import torch
    res = {}

    def pick(o):
        keep = ("value", "unit", "ms_per_step", "step_ms", "config", "roofline", "cpu_baseline", "parity", "kernels")
        return {k: o[k] for k in keep if k in o}

    a = copy.copy(args)
    a.streams, a.no_graph, a.train_step, a.group_size, a.separate_zero, a.splat_grads = 1, True, False, 0, False, False
    a.steps, a.warmup = 200, 10
    res["tiny"] = pick(bench_view(a, "tiny", headline=False))
    gc.collect(); torch.cuda.empty_cache()
    a.steps, a.warmup = 20, 3
    res["surfels"] = pick(bench_view(a, "surfels", headline=False))
    gc.collect(); torch.cuda.empty_cache()
    a.warmup = 2
    res["batch16"] = bench_batch(a, "mid", 16, 0, 3, 4, with_oracle=False)      # the oracle's time on one such view: cpu_baseline above
    gc.collect(); torch.cuda.empty_cache()
    res["large_batch8"] = bench_batch(a, "large", 8, 1024, 3, 4, with_oracle=not args.no_cpu_baseline)
    gc.collect(); torch.cuda.empty_cache()
    return res


def bench_view(args, workload, headline):
    """One view per step of `workload` through the whole path; returns the result record (the caller prints it)."""
    import numpy as np
    import torch

    from paper_2512_20017_amd import binding as B
    from paper_2512_20017_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    if workload == "mid":
        sc = synth.scene_mid(args.seed)
        cam = synth.cameras_sphere()[0]
        wl = "mid: 1M Gaussians, SH degree 3, 1920x1080, camera 0 of 16 on a radius-15 sphere"
    elif workload == "large":
        sc = synth.scene_large(args.seed)
        cam = synth.cameras_street(args.seed)[2]
        wl = "large: 8M Gaussians, SH degree 3, 3840x2160, street-level camera 2 (far plane and radius clip active)"
    elif workload == "surfels":
        sc = synth.scene_surfels(args.seed)
        cam = synth.cameras_sphere()[0]
        wl = "surfels: 1M 2D Gaussian disks, SH degree 3, 1920x1080, camera 0 of 16 on a radius-15 sphere"
    else:
        sc = synth.scene_tiny(args.seed)
        cam = synth.camera_tiny()
        wl = "tiny: 4096 Gaussians, SH degree 0, 128x128"
    surfels = workload == "surfels"
    n = int(sc["mean"].shape[0])
    W, H = cam["width"], cam["height"]
    bg = [0.0, 0.0, 0.0]
    if surfels:
        scene = B.Scene2D.from_numpy(sc)
        splats = B.Splats2D.empty(n)
        g_splats = B.SplatGrads2D.empty(n)
        alloc_ws, f_pre, f_fwd, f_bwd, f_stats = (B.alloc_workspace2d, B.pbdr2d_preprocess, B.pbdr2d_render_fwd,
                                                  B.pbdr2d_render_bwd, B.pbdr2d_render_stats)
    else:
        scene = B.Scene.from_numpy(sc)
        splats = B.Splats.empty(n)
        g_splats = B.SplatGrads.empty(n)
        alloc_ws, f_pre, f_fwd, f_bwd, f_stats = (B.alloc_workspace, B.pbdr_preprocess, B.pbdr_render_fwd,
                                                  B.pbdr_render_bwd, B.pbdr_render_stats)
    kept_groups = None
    if args.group_size > 0 and not surfels:
        ng = B.pbdr_group_count(n, args.group_size)
        g_bounds = torch.empty((7, max(ng, 1)), dtype=torch.float32, device="cuda")
        g_keep = torch.empty(max(ng, 1), dtype=torch.uint8, device="cuda")
        B.pbdr_group_bounds(scene, args.group_size, g_bounds)       # once per cloud, outside the step

        def f_pre(scene_, cam_, splats_):
            B.pbdr_preprocess_grouped(scene_, cam_, args.group_size, g_bounds, g_keep, splats_)
    grads = scene.zeros_like()
    # one fill per step where the gradient buffer is one allocation
    grad_tensors = [grads.flat] if hasattr(grads, "flat") else [v for v in vars(grads).values() if isinstance(v, torch.Tensor)]
    image = torch.empty((3, H, W), device="cuda")
    final_T = torch.empty((H, W), device="cuda")
    last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")

    # ---- size the pair capacity from one untimed pass
    cap = max(min(16 * n, 32_000_000), 1 << 16)
    ws = alloc_ws(n, W, H, cap)
    f_pre(scene, cam, splats)
    f_fwd(splats, cam, bg, cap, image, final_T, last_idx, ws)
    P, over = B.pbdr_query_lists(ws, n, W, H, cap)
    assert not over
    del ws
    cap = int(P * 1.25) + 4096
    ws = alloc_ws(n, W, H, cap)
    f_fwd(splats, cam, bg, cap, image, final_T, last_idx, ws)
    torch.cuda.synchronize()
    target = torch.from_numpy(np.ascontiguousarray(synth.target_image(args.seed, W, H).transpose(2, 0, 1))).cuda()
    dL = (torch.sign(image - target) / float(3 * W * H)).contiguous()
    n_vis = int((splats.radius > 0).sum().item())
    if args.group_size > 0 and not surfels:
        kept_groups = float(g_keep[:ng].float().mean().item())
    examined, blended = f_stats(cam, n, cap, ws)
    sum_last = int(last_idx.to(torch.int64).sum().item())

    # the step's output is dL/d(parameters); the 3D call then need not write dL/d(splat state) out (--splat-grads: do)
    g_out = g_splats if args.splat_grads else None

    def step():
        # One view per step: the backward call is the first view of its batch, so it also does the zeroing of the
        # gradient buffer (it writes every entry of every point: the view's gradient, or zero). --separate-zero clears
        # the buffer with a fill of its own first and accumulates, which leaves the same numbers.
        if args.separate_zero:
            for t in grad_tensors:
                t.zero_()
        f_pre(scene, cam, splats)
        f_fwd(splats, cam, bg, cap, image, final_T, last_idx, ws)
        f_bwd(scene, splats, cam, bg, cap, final_T, last_idx, dL, g_out, grads, ws, first_view=not args.separate_zero)

    if args.train_step:
        args.no_cpu_baseline = True      # the parameters move: the oracle legs below describe the fixed scene only
        assert not surfels, "--train-step is wired for the 3D Gaussian workloads"
        m1, m2 = scene.zeros_like(), scene.zeros_like()
        visible = torch.zeros(n, dtype=torch.uint8, device="cuda")
        loss = torch.zeros(1, device="cuda")
        lrs = dict(mean=1.6e-4, log_scale=5e-3, quat=1e-3, logit=5e-2, sh=2.5e-3)
        it = [0]

        def step():   # noqa: F811  (one view per iteration: its backward call writes the whole gradient buffer)
            it[0] += 1
            f_pre(scene, cam, splats)
            if args.unfused_adam:
                visible.zero_()
                B.pbdr_mark_visible(splats.radius, visible)
            f_fwd(splats, cam, bg, cap, image, final_T, last_idx, ws)
            B.pbdr_l1_loss(image, target, loss, dL)
            if not args.unfused_adam:
                # compositing backward stops at dL/d(splat state); the splatting backward and the Adam step are one pass
                f_bwd(None, splats, cam, bg, cap, final_T, last_idx, dL, g_splats, None, ws)
                B.pbdr_preprocess_bwd_batch_adam(scene, [cam], [splats], [g_splats], m1, m2, list(lrs.values()), 0.9, 0.999,
                                                 1e-15, it[0])
                return
            f_bwd(scene, splats, cam, bg, cap, final_T, last_idx, dL, g_out, grads, ws, first_view=not args.separate_zero)
            for k, lr in lrs.items():
                B.pbdr_adam_selective(getattr(scene, k), getattr(grads, k), getattr(m1, k), getattr(m2, k), visible,
                                      lr, 0.9, 0.999, 1e-15, it[0], zero_grad=args.separate_zero)
        for t in grad_tensors:
            t.zero_()

    # a plain device copy as the yardstick for the HBM-bound kernels: 256 MiB read + 256 MiB written, timed with events
    copy_gbs = None
    if headline and not args.train_step:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    names = B.profile_kernel_names()
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()

    # ---- untimed profiling pass over every kernel: which one dominates?
    prof_steps = 3
    B.pbdr_profile_begin((1 << len(names)) - 1, 256 * prof_steps)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    per_kernel = {}
    for kid, name in enumerate(names):
        ms, cnt = B.pbdr_profile_collect(kid)
        if cnt:
            per_kernel[name] = dict(ms_per_step=ms / prof_steps, launches_per_step=cnt / prof_steps)
    B.pbdr_profile_end()
    dominant = max(per_kernel, key=lambda k: per_kernel[k]["ms_per_step"])
    dom_id = names.index(dominant)

    # ---- timed region: K steps, only the dominant kernel carries events
    B.pbdr_profile_begin(1 << dom_id, 64 * args.steps + 64)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms, dom_cnt = B.pbdr_profile_collect(dom_id)
    B.pbdr_profile_end()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    views_per_s = args.steps / (t1 - t0)
    dom_avg_ms = dom_ms / max(dom_cnt, 1)
    # the spread of single steps: one event pair per step, outside the kernels (>= 20 steps), after the timed region
    step_ms = spread(per_step_times(torch, step, max(20, min(args.steps, 100))))

    # ---- roofline of the dominant kernel
    K = (scene.sh_degree + 1) ** 2
    tile_passes = max(1, (max(1, (((W + 15) // 16) * ((H + 15) // 16) - 1).bit_length()) + 7) // 8)
    hbm_bytes = {   # algorithmic bytes per step
        "k_preprocess": 16.0 * n + (32.0 + 12.0 * K + 40.0) * n_vis,
        "k_count_visible": 8.0 * n + 8.0 * n_vis,
        "k_pack_dup": 4.0 * n + (44.0 + 64.0) * n_vis + 8.0 * P,
        "k_radix_hist": tile_passes * 4.0 * P,
        "k_radix_scatter": tile_passes * 16.0 * P,
        "k_tile_ranges": 4.0 * P,
        "k_tile_depth_sort": 12.0 * P,
        "k_gather_splat_grads": 8.0 * n + 48.0 * P + 36.0 * n,
        # accumulate: read + write of the visible points' gradient entries; first view: one write of every point's
        "k_preprocess_bwd": 4.0 * n + (36.0 + 32.0 + 12.0 * K) * n_vis
                            + ((44.0 + 12.0 * K) * 2 * n_vis if args.separate_zero else (44.0 + 12.0 * K) * n),
        "k_l1_loss": 36.0 * W * H,                                        # two reads, one write per value
        "k_adam_selective": (11 + 3 * K) * (1.0 * n + 32.0 * n_vis),      # mask byte per point and plane; 4 reads + 4 writes
    }
    alu_flops = {
        "k_composite_fwd": FWD_FLOPS_PER_EXAMINED * examined + FWD_FLOPS_PER_BLENDED * blended,
        "k_composite_bwd": BWD_FLOPS_PER_EXAMINED * sum_last + BWD_FLOPS_PER_BLENDED * blended,
    }
    if surfels:   # same kernel ids, the surfel kernels behind them; only the compositing figures are stated
        hbm_bytes = {}
        alu_flops = {
            "k_composite_fwd": FWD2D_FLOPS_PER_EXAMINED * examined + FWD_FLOPS_PER_BLENDED * blended,
            "k_composite_bwd": FWD2D_FLOPS_PER_EXAMINED * sum_last + BWD2D_FLOPS_PER_BLENDED * blended,
        }
    if dominant in alu_flops:
        ach = alu_flops[dominant] / (dom_avg_ms * 1e-3) / 1e12
        roofline = dict(kernel=dominant, bound="alu", achieved=ach, peak=ALU_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=ach / ALU_PEAK_TFLOPS, traffic=None, avg_launch_ms=dom_avg_ms, launches_timed=dom_cnt,
                        flops_per_launch=alu_flops[dominant])
    elif dominant in hbm_bytes:
        ach = hbm_bytes[dominant] / (dom_ms / args.steps * 1e-3) / 1e9
        roofline = dict(kernel=dominant, bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=ach / HBM_PEAK_GBS, traffic=None, avg_launch_ms=dom_avg_ms, launches_timed=dom_cnt,
                        bytes_per_launch=hbm_bytes[dominant])
    else:
        roofline = dict(kernel=dominant, bound="hbm", achieved=None, peak=HBM_PEAK_GBS, unit="GB/s", frac=None,
                        traffic=None, avg_launch_ms=dom_avg_ms, launches_timed=dom_cnt)
    if workload == "mid":
        roofline["traffic"] = profiled_traffic(dominant)
        # share of the vector ALU's issue capacity (1024 SIMDs x 2.4 GHz x duration) that the compositing kernels' counted
        # instructions take, next to the flop fraction: counters of the committed profile, durations of this run
        issue = {}
        for kname in ("k_composite_fwd", "k_composite_bwd"):
            cyc = profiled_valu_cycles(kname)
            if cyc and kname in per_kernel:
                t_k = dom_avg_ms if kname == dominant else per_kernel[kname]["ms_per_step"] / per_kernel[kname]["launches_per_step"]
                issue[kname] = cyc / (1024 * 2.4e9 * t_k * 1e-3)
        roofline["valu_issue_frac"] = issue.get(dominant)
        roofline["valu_issue_frac_by_kernel"] = issue
    for name, rec in per_kernel.items():
        t = rec["ms_per_step"] * 1e-3
        if name in alu_flops:
            rec["tflops"] = alu_flops[name] / t / 1e12
        elif name in hbm_bytes:
            rec["gbs"] = hbm_bytes[name] / t / 1e9

    # ---- CPU oracle on the host cores: one full view of the same workload (forward + backward)
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        cpu, parity, rf = oracle_view_check(np, oracle, sc, cam, splats.to_numpy(), image, P, bg, dL, surfels=surfels)
        ok = rf["fragile"] == 0
        parity.update(examined_gpu=int(examined), blended_gpu=int(blended),
                      last_idx_mismatch=int((last_idx.cpu().numpy().astype(np.uint32) != rf["last_idx"])[ok].sum()))

    # ---- the same step with several views in flight (not `value`): every view has its own splat state, workspace and
    # outputs and runs on its own stream, so one view's short launch-bound kernels (binning, sort) fill the gaps of
    # another's compositing kernels. Per-kernel durations stretch under sharing, which is why the roofline above is
    # taken with one view in flight.
    overlapped = None
    if headline and args.streams > 1 and not args.train_step and not surfels:
        ctxs = []
        for _ in range(args.streams):
            ctxs.append(dict(stream=torch.cuda.Stream(), splats=B.Splats.empty(n), g2=B.SplatGrads.empty(n), grads=scene.zeros_like(),
                             image=torch.empty((3, H, W), device="cuda"), final_T=torch.empty((H, W), device="cuda"),
                             last_idx=torch.empty((H, W), dtype=torch.int32, device="cuda"), ws=alloc_ws(n, W, H, cap)))
        torch.cuda.synchronize()

        def step_on(c):
            with torch.cuda.stream(c["stream"]):
                f_pre(scene, cam, c["splats"])
                f_fwd(c["splats"], cam, bg, cap, c["image"], c["final_T"], c["last_idx"], c["ws"])
                f_bwd(scene, c["splats"], cam, bg, cap, c["final_T"], c["last_idx"], dL, c["g2"] if args.splat_grads else None,
                      c["grads"], c["ws"], first_view=True)

        for i in range(2 * args.streams):
            step_on(ctxs[i % args.streams])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_on(ctxs[i % args.streams])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # same results as the one-view-in-flight run: the image bit for bit; the gradient to the rounding of the
        # backward kernel's LDS adds, whose order among a tile's four wavefronts is not fixed
        same_image = all(torch.equal(c["image"], image) for c in ctxs)
        gscale = float(grads.flat.abs().max().item())
        gdiff = max(float((c["grads"].flat - grads.flat).abs().max().item()) for c in ctxs) / max(gscale, 1e-30)
        overlapped = dict(views_in_flight=args.streams, views_per_s=args.steps / (t1 - t0),
                          ms_per_view=(t1 - t0) * 1e3 / args.steps, image_bitwise_equal=same_image,
                          max_gradient_diff_rel_to_max=gdiff)
        del ctxs

    # ---- the same step recorded once into a HIP graph and replayed (not `value`): the calls are kernel launches on the
    # caller's stream and nothing else, so the step can be captured; one graph launch then stands for its ~45 launches
    graph_replay = None
    if headline and not args.no_graph and not args.train_step:
        graph = torch.cuda.CUDAGraph()
        before = grads.flat.clone() if hasattr(grads, "flat") else None
        with torch.cuda.graph(graph):
            step()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        graph_replay = dict(views_per_s=args.steps / (t1 - t0), ms_per_step=(t1 - t0) * 1e3 / args.steps)
        if before is not None:
            gscale = float(before.abs().max().item())
            graph_replay["max_gradient_diff_rel_to_max"] = float((grads.flat - before).abs().max().item()) / max(gscale, 1e-30)
        del graph

    out = {
        "metric": "training iterations/sec (splat, render, L1 loss, backward, selective Adam), one view" if args.train_step else
                  {"mid": "fwd+bwd views/sec at 1080p, 1M Gaussians",
                   "surfels": "fwd+bwd views/sec at 1080p, 1M 2D Gaussian surfels",
                   "large": "fwd+bwd views/sec at 4K, 8M Gaussians, street view"}.get(workload, "fwd+bwd views/sec"),
        "value": views_per_s, "unit": "views/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "step_ms": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl, "n_gaussians": n, "width": W, "height": H, "sh_degree": scene.sh_degree,
                   "visible": n_vis, "tile_pairs": int(P), "pairs_examined_fwd": int(examined),
                   "pairs_examined_bwd": sum_last, "pairs_blended": int(blended), "seed": args.seed,
                   "group_size": args.group_size, "groups_kept": kept_groups},
        "mpixel_per_s": views_per_s * W * H / 1e6,
        "device_copy_gbs": copy_gbs,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": per_kernel,
        "parity": parity,
        "overlapped": overlapped,
        "graph_replay": graph_replay,
    }
    return out


if __name__ == "__main__":
    main()
