#!/usr/bin/env python3
"""Benchmark of the lowering-based convolutional layer on one MI355X.

Default mode.  One "step" = the whole hot path over one batch: forward, backward-data and
backward-weights of CaffeNet conv1..conv5 at batch 256 (15 passes; lowering, multiply and
lifting all inside the timed region; inputs, weights, upstream gradients and the workspace
already resident in HBM).  Prints ONE JSON line with the headline metric (algorithmic conv
GFLOP/s), the spread of the per-step times, the roofline figures of the dominant kernel
(measured with HIP events on the launching stream), the rates of the lowering / lifting kernels
of the materialised layouts (a short extra leg that forces Types 1, 2 and 3) and the CPU
oracle's rate on a bounded sample of the same workload.

Other modes (tables on stdout, meant to be kept under profiles/):
  --config sweep      the channel-ratio study (Appendix A): batch 128, 28x28, k in {1,3}, six
                      (C,O) pairs, forward pass, Types 1/2/3, the fused layout and AUTO timed.
  --config batching   the batching study (Sec. 2.2): Type 1 forced, the whole step run with
                      1 .. N images per lowered matrix.
  --config e2e        one training iteration of CaffeNet (conv, ReLU, pooling, normalisation, fully
                      connected, dropout, softmax loss; no weight update), with the share of time
                      per kind of layer (Sec. 1 and 3.2 of the paper time whole iterations).
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_caffenet_b256_f32.txt")
STREAM_KERNELS = ("lower_kernel", "lower_direct_kernel", "lift_kernel", "inv_lift_kernel",
                  "inv_lift_direct_kernel", "inv_lower_kernel")


def measured_traffic(kernel):
    """(HBM bytes per launch of `kernel`, provenance) from the committed rocprofv3 --pmc summary;
    (None, reason) when the file is absent, was taken from other kernel sources, or has no row for
    this kernel."""
    from paper_1504_04343_amd.profile_summary import kernel_sources_digest
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None, "no counter profile"
    digest = None
    for line in lines:
        if line.startswith("# kernel sources digest:"):
            digest = line.split(":", 1)[1].strip()
    if digest != kernel_sources_digest():
        return None, "counter profile was taken from other kernel sources (%s)" % digest
    for line in lines:
        f = line.split("\t")
        if not line.startswith("#") and len(f) >= 2 and f[0] == kernel:
            return int(f[1]), "profiles/%s, kernel sources %s" % (os.path.basename(TRAFFIC_FILE), digest)
    return None, "kernel not in the counter profile"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", choices=["caffenet", "sweep", "batching", "e2e"], default="caffenet")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--precision", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--lowering", type=int, default=0, help="0 = auto (default), 1..4 = force")
    ap.add_argument("--chunk", type=int, default=0, help="images per chunk (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap-leg", action="store_true",
                    help="skip the leg that repeats the steps with backward-weights on a second stream")
    ap.add_argument("--no-stream-leg", action="store_true",
                    help="skip the extra leg that times the lowering / lifting kernels")
    ap.add_argument("--stream-leg-only", action="store_true",
                    help="run only the leg that times the lowering / lifting kernels (for profilers)")
    ap.add_argument("--stream-leg-type", type=int, default=0,
                    help="with --stream-leg-only: force this materialised layout only (0 = all three)")
    ap.add_argument("--cpu-sample-images", type=int, default=64)
    ap.add_argument("--per-kernel", action="store_true", help="also print the per-kernel table")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain 1 GiB device copy (reference row for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE scaling)")
    return ap.parse_args()


class Stack:
    """Resident tensors of a list of layers and one workspace that fits every pass."""

    def __init__(self, B, synth, layers, lowering, prec, chunk):
        import torch
        self.B, self.layers = B, layers
        self.passes = [B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS]
        self.state, ws_bytes = [], 0
        for L in layers:
            d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, lowering, prec)
            t = dict(L=L, d=d,
                     x=torch.from_numpy(synth.make_x(L)).cuda(), w=torch.from_numpy(synth.make_w(L)).cuda(),
                     b=torch.from_numpy(synth.make_bias(L)).cuda(), dy=torch.from_numpy(synth.make_dy(L)).cuda())
            t["y"] = torch.empty_like(t["dy"])
            t["dx"] = torch.empty_like(t["x"])
            t["dw"] = torch.empty_like(t["w"])
            t["db"] = torch.empty_like(t["b"])
            t["picked"] = {p: (lowering or B.cct_pick_lowering(d, p)) for p in self.passes}
            for p in self.passes:
                n = B.cct_conv_workspace_bytes(d, p) if not chunk else \
                    B.cct_conv_workspace_bytes_for_chunk(d, p, min(chunk, L.N))
                ws_bytes = max(ws_bytes, n)
            self.state.append(t)
        self.ws_bytes = ws_bytes
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        self.flops_per_step = sum(L.flops for L in layers) * len(self.passes)

    def step(self):
        B, ws = self.B, self.ws
        for t in self.state:
            d = t["d"]
            B.cct_conv_forward(d, t["x"], t["w"], t["b"], t["y"], ws)
            B.cct_conv_backward_data(d, t["w"], t["dy"], t["dx"], ws)
            B.cct_conv_backward_weights(d, t["x"], t["dy"], t["dw"], t["db"], ws)

    def overlapped_step_fn(self):
        """The same 15 passes in training order, with the one overlap a training step allows inside a
        layer: backward-weights of a layer does not depend on its backward-data, so it goes to a
        second stream (default priority) with a workspace of its own."""
        import torch
        B = self.B
        ws2 = torch.empty_like(self.ws)
        side = torch.cuda.Stream()

        def step():
            main = torch.cuda.current_stream()
            for t in self.state:
                B.cct_conv_forward(t["d"], t["x"], t["w"], t["b"], t["y"], self.ws)
            side.wait_stream(main)
            for t in reversed(self.state):
                B.cct_conv_backward_data(t["d"], t["w"], t["dy"], t["dx"], self.ws)
                with torch.cuda.stream(side):
                    B.cct_conv_backward_weights(t["d"], t["x"], t["dy"], t["dw"], t["db"], ws2)
            main.wait_stream(side)
        return step


def time_steps(step, steps, warmup):
    """(wall seconds for `steps` steps, list of per-step GPU milliseconds).  The wall clock brackets
    all steps between two synchronisations; the per-step figures come from events recorded between
    the steps on the same stream, so they add no host synchronisation."""
    import torch
    for _ in range(warmup):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    return elapsed, [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]


def spread(per_step_ms):
    mean = statistics.fmean(per_step_ms)
    sd = statistics.pstdev(per_step_ms) if len(per_step_ms) > 1 else 0.0
    return {"median_ms": round(statistics.median(per_step_ms), 3), "min_ms": round(min(per_step_ms), 3),
            "max_ms": round(max(per_step_ms), 3), "cv": round(sd / mean, 4) if mean else None}


def profiled(B, step, steps):
    import torch
    B.cct_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    B.cct_profile_enable(False)
    return B.cct_profile_read(64)


def stream_kernel_leg(B, synth, batch, prec, steps=2, types=(1, 2, 3)):
    """Rates of the lowering / lifting kernels and their adjoints: AUTO runs most passes fused, so
    they are timed in a leg of their own that forces each materialised layout (a layout the cost
    model prices at more than 5x the cheapest for a layer and pass is skipped: Type 3 of conv1
    would need hundreds of GB).  Algorithmic bytes = tensor once + matrix once."""
    import torch
    out = {}
    agg = {}
    for lowering in types:
        for L in synth.caffenet(batch):
            d0 = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, 0, prec)
            d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, lowering, prec)
            x = torch.from_numpy(synth.make_x(L)).cuda()
            w = torch.from_numpy(synth.make_w(L)).cuda()
            dy = torch.from_numpy(synth.make_dy(L)).cuda()
            y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
            for p in (B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS):
                try:
                    costs = []
                    for t in (1, 2, 3, 4):
                        try:
                            costs.append(B.cct_lowering_cost(d0, p, t))
                        except B.CctError:
                            pass
                    if B.cct_lowering_cost(d0, p, lowering) > 5 * min(costs):
                        continue
                    ws = B.alloc_workspace(d, p)
                except B.CctError:
                    continue

                def run():
                    if p == B.PASS_FORWARD:
                        B.cct_conv_forward(d, x, w, None, y, ws)
                    elif p == B.PASS_BACKWARD_DATA:
                        B.cct_conv_backward_data(d, w, dy, dx, ws)
                    else:
                        B.cct_conv_backward_weights(d, x, dy, dw, None, ws)
                run()
                for e in profiled(B, run, steps):
                    if e["name"].startswith(STREAM_KERNELS):
                        key = e["name"].split("<")[0].replace("_direct", "")
                        a = agg.setdefault(key, [0.0, 0.0, 0])
                        a[0] += e["bytes"]
                        a[1] += e["total_ms"]
                        a[2] += e["launches"]
                del ws
            del x, w, dy, y, dx, dw
    for k, (nbytes, ms, n) in sorted(agg.items()):
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[k] = {"GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4), "launches": n,
                  "algorithmic_MB_per_launch": round(nbytes / n / 1e6, 1), "avg_launch_ms": round(ms / n, 4)}
    return out


def run_caffenet(args, B, synth, torch):
    batch = args.batch or 256
    prec = B.PREC_F32 if args.precision == "f32" else B.PREC_BF16_IN_F32_ACC
    layers = synth.caffenet(batch)
    st = Stack(B, synth, layers, args.lowering, prec, args.chunk)
    elapsed, per_step = time_steps(st.step, args.steps, args.warmup)
    ms_per_step = elapsed / args.steps * 1e3
    gflops = st.flops_per_step / 1e9 / (elapsed / args.steps)

    # ---- per-kernel HIP-event timing over the same steps (second leg, same launches) --------
    prof = profiled(B, st.step, args.steps)
    total_kernel_ms = sum(e["total_ms"] for e in prof)

    def is_mfma(e):   # the GEMMs and the fused conv kernels (matrix-core bound); the rest stream
        return e["name"].startswith(("gemm_", "conv_fused", "conv_bwdw_fused"))
    gemms = [e for e in prof if is_mfma(e)]
    dom = max(gemms, key=lambda e: e["total_ms"])
    avg_ms = dom["total_ms"] / dom["launches"]
    achieved_tflops = dom["flops"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
    peak = PEAK_FP32_MFMA_TFLOPS if args.precision == "f32" else PEAK_BF16_MFMA_TFLOPS
    headline = args.precision == "f32" and batch == 256 and not args.lowering and not args.chunk
    traffic, traffic_src = measured_traffic(dom["name"]) if headline else (None, "not the headline configuration")
    roofline = {
        "bound": "mfma", "kernel": dom["name"], "achieved": round(achieved_tflops, 2), "peak": peak,
        "unit": "TFLOP/s", "frac": round(achieved_tflops / peak, 4),
        "traffic": traffic, "traffic_source": traffic_src,
        "algorithmic_bytes_per_launch": int(dom["bytes"] / dom["launches"]),
        "avg_launch_ms": round(avg_ms, 4), "launches_per_step": dom["launches"] / args.steps,
        "share_of_step_kernel_time": round(dom["total_ms"] / total_kernel_ms, 3),
    }
    if args.precision != "f32" and not dom["name"].startswith("conv_fused"):
        # bf16 matrix cores are 16x the fp32 ones: a GEMM on bf16 lowered matrices is bound by
        # streaming those matrices, so it is quoted against the HBM roof (the fused bf16 kernel,
        # which has no such matrices, stays a contraction quoted against the bf16 matrix peak)
        gbs = dom["bytes"] / dom["launches"] / (avg_ms * 1e-3) / 1e9
        roofline.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(gbs / PEAK_HBM_GBS, 4), "mfma_tflops": round(achieved_tflops, 2),
                         "mfma_frac_of_bf16_peak": round(achieved_tflops / peak, 4)})
    all_gemm_flops = sum(e["flops"] for e in gemms)
    all_gemm_ms = sum(e["total_ms"] for e in gemms)
    # the lowering / lifting kernels that the timed step itself runs
    streams = [e for e in prof if e["name"].startswith(STREAM_KERNELS)]
    stream_bytes = sum(e["bytes"] for e in streams)
    stream_ms = sum(e["total_ms"] for e in streams)
    pname = "fp32" if args.precision == "f32" else "bf16"
    phases = {
        "all_gemm_tflops": round(all_gemm_flops / (all_gemm_ms * 1e-3) / 1e12, 2),
        "all_gemm_frac_of_%s_mfma_peak" % pname: round(all_gemm_flops / (all_gemm_ms * 1e-3) / 1e12 / peak, 4),
        "gemm_share_of_kernel_time": round(all_gemm_ms / total_kernel_ms, 3),
        "lower_lift_GBps": round(stream_bytes / (stream_ms * 1e-3) / 1e9, 1) if stream_ms else None,
        "lower_lift_frac_of_hbm_peak":
            round(stream_bytes / (stream_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if stream_ms else None,
        "lower_lift_share_of_kernel_time": round(stream_ms / total_kernel_ms, 3),
    }
    if args.per_kernel:
        for e in sorted(prof, key=lambda e: -e["total_ms"]):
            ms = e["total_ms"] / e["launches"]
            print("# %-40s launches/step %5.1f  avg %8.4f ms  %8.2f TFLOP/s  %8.1f GB/s  share %.3f" % (
                e["name"], e["launches"] / args.steps, ms, e["flops"] / e["launches"] / ms / 1e9,
                e["bytes"] / e["launches"] / ms / 1e6, e["total_ms"] / total_kernel_ms), file=sys.stderr)
    picked = {t["L"].name: [t["picked"][p] for p in st.passes] for t in st.state}
    ws_mib = st.ws_bytes >> 20

    # ---- CPU oracle on a bounded sample of the same workload --------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_images, batch)
        cpu_flops, cpu_s = 0.0, 0.0
        for t in st.state:
            L = t["L"].with_batch(ns)
            od = oracle.Dims(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups)
            x = t["x"][:ns].cpu().numpy()
            w = t["w"].cpu().numpy()
            b = t["b"].cpu().numpy()
            dy = t["dy"][:ns].cpu().numpy()
            c0 = time.perf_counter()
            oracle.conv_forward(od, x, w, b)
            oracle.conv_backward_data(od, w, dy)
            oracle.conv_backward_weights(od, x, dy)
            cpu_s += time.perf_counter() - c0
            cpu_flops += 3 * L.flops
        cpu = {"value": round(cpu_flops / 1e9 / cpu_s, 2), "unit": "GFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "conv1-5 forward+backward-data+backward-weights on the first %d images of the "
                         "batch (%.1f GFLOP, %.1f s)" % (ns, cpu_flops / 1e9, cpu_s)}

    # ---- the same steps with backward-weights overlapping backward-data (own leg) ------------
    overlap = None
    if not args.no_overlap_leg:
        o_elapsed, o_per_step = time_steps(st.overlapped_step_fn(), args.steps, args.warmup)
        overlap = {"what": "same 15 passes per step; backward-weights of each layer on a second stream, "
                           "concurrent with its backward-data (reported beside `value`, never as it)",
                   "streams": 2, "ms_per_step": round(o_elapsed / args.steps * 1e3, 3),
                   "value": round(st.flops_per_step / 1e9 / (o_elapsed / args.steps), 1), "unit": "GFLOP/s",
                   "step_time_spread": spread(o_per_step)}

    # ---- the lowering / lifting kernels of the materialised layouts (own leg) ---------------
    if not args.no_stream_leg and headline:
        flops_per_step = st.flops_per_step
        del st
        torch.cuda.empty_cache()
        phases["materialised_layout_kernels"] = stream_kernel_leg(B, synth, batch, prec)
    else:
        flops_per_step = st.flops_per_step

    out = {
        "metric": "conv GFLOP/s fwd+bwd, CaffeNet conv1-5 batch 256; % fp32 MFMA peak",
        "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.precision == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": "CaffeNet conv1-5 forward + backward-data + backward-weights, batch %d, "
                               "fp32, auto lowering" % batch if args.precision == "f32" and not args.lowering
                   else "CaffeNet conv1-5, batch %d, precision %s, lowering %d, passes 3" % (
                       batch, args.precision, args.lowering),
                   "batch": batch, "gflop_per_step": round(flops_per_step / 1e9, 2),
                   "lowering_picked": picked,
                   "workspace_MiB": ws_mib,
                   "frac_of_%s_mfma_peak" % pname:
                       round(gflops / 1e3 / (PEAK_FP32_MFMA_TFLOPS if args.precision == "f32"
                                             else PEAK_BF16_MFMA_TFLOPS), 4)},
        "step_time_spread": spread(per_step),
        "roofline": roofline,
        "phases": phases,
        "two_stream_step": overlap,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def time_forward(B, torch, L, synth, lowering, reps):
    """Median milliseconds of the forward pass of one layer with one layout (events on the stream)."""
    d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, lowering)
    x = torch.from_numpy(synth.make_x(L)).cuda()
    w = torch.from_numpy(synth.make_w(L)).cuda()
    b = torch.from_numpy(synth.make_bias(L)).cuda()
    y = torch.empty((L.N, L.O, L.Hout, L.Wout), device="cuda")
    ws = B.alloc_workspace(d, B.PASS_FORWARD)
    for _ in range(2):
        B.cct_conv_forward(d, x, w, b, y, ws)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record()
    for i in range(reps):
        B.cct_conv_forward(d, x, w, b, y, ws)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))


def run_sweep(args, B, synth, torch):
    """Appendix A on MI355X: which layout wins as #input/#output channels varies, and what the
    optimizer picks.  One line per shape; regret = time(pick) / time(best) - 1."""
    batch = args.batch or 128
    reps = max(5, args.steps)
    print("# lowering trade-off sweep, forward pass, batch %d, 28x28, fp32; median of %d runs, ms" % (batch, reps))
    print("# %-24s %8s %8s %8s %8s %8s   %-5s %-5s %7s" % (
        "shape (k, C->O)", "type1", "type2", "type3", "fused", "auto", "pick", "best", "regret"))
    worst = 0.0
    rows = []
    for L in synth.tradeoff_sweep(batch):
        times = {}
        for t in (1, 2, 3, 4, 0):
            try:
                times[t] = time_forward(B, torch, L, synth, t, reps)
            except B.CctError:
                times[t] = None
        d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups)
        pick = B.cct_pick_lowering(d, B.PASS_FORWARD)
        forced = {t: v for t, v in times.items() if t and v is not None}
        best = min(forced, key=forced.get)
        regret = forced[pick] / forced[best] - 1.0
        worst = max(worst, regret)
        rows.append(dict(shape=L.name, ms={str(k): v for k, v in times.items()}, pick=pick, best=best,
                         regret=round(regret, 4)))
        fmt = lambda v: "%8.3f" % v if v is not None else "%8s" % "-"
        print("  %-24s %s %s %s %s %s   %-5d %-5d %6.1f%%" % (
            "k%d %4d->%-4d" % (L.K, L.C, L.O), fmt(times[1]), fmt(times[2]), fmt(times[3]), fmt(times[4]),
            fmt(times[0]), pick, best, 100 * regret))
    print("# worst regret of the optimizer's pick: %.1f%%" % (100 * worst))
    print(json.dumps({"config": "sweep", "batch": batch, "worst_regret": round(worst, 4), "rows": rows}))


def run_batching(args, B, synth, torch):
    """Sec. 2.2 on the GPU: Type 1 (the layout Caffe uses one image at a time) forced for all 15
    passes, every pass given a workspace for c images, so lowering, GEMM and lifting run on c
    images at a time; last row = AUTO with the default workspace."""
    batch = args.batch or 256
    steps = max(3, min(args.steps, 10))
    print("# batching study, CaffeNet conv1-5 fwd+bwd, batch %d, fp32: images per lowered matrix vs step time" % batch)
    print("# %-18s %10s %10s %12s %14s %12s" % ("images per GEMM", "ms/step", "TFLOP/s", "GEMM TFLOP/s",
                                                 "lower/lift GB/s", "workspace MiB"))
    chunks = [c for c in (1, 4, 16, 32, 64, 128, 256, 512, 1024) if c <= batch]
    rows = []
    for c in chunks + [0]:
        st = Stack(B, synth, synth.caffenet(batch), 1 if c else 0, B.PREC_F32, c)
        elapsed, _ = time_steps(st.step, steps if c != 1 else 2, 1)
        n = steps if c != 1 else 2
        prof = profiled(B, st.step, 1)
        g = [e for e in prof if e["name"].startswith(("gemm_", "conv_fused", "conv_bwdw_fused"))]
        s = [e for e in prof if e["name"].startswith(STREAM_KERNELS)]
        gt = sum(e["flops"] for e in g) / (sum(e["total_ms"] for e in g) * 1e-3) / 1e12
        sb = sum(e["bytes"] for e in s) / (sum(e["total_ms"] for e in s) * 1e-3) / 1e9 if s else float("nan")
        ms = elapsed / n * 1e3
        rows.append(dict(chunk=c, ms_per_step=round(ms, 3), tflops=round(st.flops_per_step / 1e9 / ms, 2),
                         workspace_MiB=st.ws_bytes >> 20))
        print("  %-18s %10.2f %10.1f %12.1f %14.0f %12d" % (
            ("%d" % c) if c else "AUTO (fused)", ms, st.flops_per_step / 1e9 / ms, gt, sb, st.ws_bytes >> 20))
        del st
        torch.cuda.empty_cache()
    print(json.dumps({"config": "batching", "batch": batch, "rows": rows}))


def run_e2e(args, B, synth, torch):
    """One training iteration of CaffeNet: conv1-5 with ReLU, three max-pooling and two normalisation
    layers, fc6-8 through the convolution entry points with ReLU and dropout (ratio 0.5, a fixed
    seeded mask) after fc6 and fc7, the softmax loss on seeded labels; forward and backward (conv1's
    input gradient is not needed and not computed; no weight update), batch 256.  The analogue of the paper's end-to-end timing (Sec. 3.2) and of its remark that the
    convolutional layers take 70-90 % of the time (Sec. 1): per-kind shares from HIP events around
    every call of a second, separately run, instrumented iteration."""
    N = args.batch or 256
    prec = B.PREC_F32 if args.precision == "f32" else B.PREC_BF16_IN_F32_ACC
    convs = synth.caffenet(N)
    fcs = [synth.Layer("fc6", N, 256, 6, 6, 4096, 6, 1, 0, 1, "relu_normal", 0.005, 0.0),
           synth.Layer("fc7", N, 4096, 1, 1, 4096, 1, 1, 0, 1, "relu_normal", 0.005, 0.0),
           synth.Layer("fc8", N, 4096, 1, 1, 1000, 1, 1, 0, 1, "relu_normal", 0.01, 0.0)]
    pool_after = {"conv1": 55, "conv2": 27, "conv5": 13}
    norm_after = ("conv1", "conv2")
    dev = "cuda"
    net, ws_bytes = [], 0
    for L in convs + fcs:
        d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, 0, prec)
        t = dict(L=L, d=d, kind="fc" if L.name.startswith("fc") else "conv",
                 w=torch.from_numpy(synth.make_w(L)).cuda(), b=torch.from_numpy(synth.make_bias(L)).cuda(),
                 y=torch.empty((N, L.O, L.Hout, L.Wout), device=dev))
        t["dw"], t["db"] = torch.empty_like(t["w"]), torch.empty_like(t["b"])
        t["gy"] = torch.empty_like(t["y"])              # gradient at the layer's output (before ReLU)
        if L.name != "fc8":
            t["a"] = torch.empty_like(t["y"])           # after ReLU
            t["ga"] = torch.empty_like(t["y"])
        if L.name in pool_after:
            H = pool_after[L.name]
            pd = B.make_pool_desc(N, L.O, H, H, 3, 2, 0)
            ho, wo = B.cct_pool_output_dims(pd)
            t.update(pd=pd, p=torch.empty((N, L.O, ho, wo), device=dev),
                     am=torch.empty((N, L.O, ho, wo), dtype=torch.int32, device=dev))
            t["gp"] = torch.empty_like(t["p"])
            if L.name in norm_after:
                t.update(ld=B.make_lrn_desc(N, L.O, ho, wo), n=torch.empty_like(t["p"]), gn=torch.empty_like(t["p"]))
        if L.name in ("fc6", "fc7"):
            keep = np.random.default_rng(len(net)).random((N, L.O, 1, 1)) >= 0.5
            t.update(dm=torch.from_numpy(keep.astype(np.uint8)).cuda(), do=torch.empty_like(t["y"]))
        for p_ in (B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS):
            ws_bytes = max(ws_bytes, B.cct_conv_workspace_bytes(d, p_))
        net.append(t)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    x0 = torch.from_numpy(synth.make_x(convs[0])).cuda()
    label = torch.from_numpy(np.random.default_rng(7).integers(0, 1000, N).astype(np.int32)).cuda()
    prob = torch.empty((N, 1000), device=dev)
    image_loss, loss = torch.empty(N, device=dev), torch.empty(1, device=dev)
    for i, t in enumerate(net):                       # wire inputs and input gradients
        t["x"] = x0 if i == 0 else net[i - 1]["out"]
        t["out"] = t.get("do", t.get("n", t.get("p", t.get("a", t["y"]))))
        if t["L"].name == "fc6":
            t["x"] = t["x"].view(N, 256, 6, 6)
        t["gx"] = None if i == 0 else torch.empty_like(t["x"])
    flops = sum(3 * t["L"].flops for t in net) - convs[0].flops

    def iteration(tick=lambda kind: None):
        for t in net:                                  # ---- forward
            B.cct_conv_forward(t["d"], t["x"], t["w"], t["b"], t["y"], ws); tick(t["kind"])
            if "a" in t:
                B.cct_relu_forward(t["y"], t["a"]); tick("relu")
            if "pd" in t:
                B.cct_maxpool_forward(t["pd"], t["a"], t["p"], t["am"]); tick("pool")
            if "ld" in t:
                B.cct_lrn_forward(t["ld"], t["p"], t["n"]); tick("norm")
            if "dm" in t:
                B.cct_dropout_forward(t["a"], t["dm"], 2.0, t["do"]); tick("drop")
        B.cct_softmax_loss_forward(net[-1]["y"].view(N, 1000), label, prob, image_loss, loss); tick("loss")
        g = net[-1]["gy"]
        B.cct_softmax_loss_backward(prob, label, g.view(N, 1000)); tick("loss")
        for i in range(len(net) - 1, -1, -1):          # ---- backward
            t = net[i]
            if "dm" in t:
                B.cct_dropout_backward(g.view_as(t["do"]), t["dm"], 2.0, t["ga"]); tick("drop"); g = t["ga"]
            if "ld" in t:
                B.cct_lrn_backward(t["ld"], t["p"], g, t["gn"]); tick("norm"); g = t["gn"]
            if "pd" in t:
                B.cct_maxpool_backward(t["pd"], g.view_as(t["p"]), t["am"], t["ga"]); tick("pool"); g = t["ga"]
            if "a" in t:
                B.cct_relu_backward(t["y"], g.view_as(t["y"]), t["gy"]); tick("relu"); g = t["gy"]
            g = g.view_as(t["y"])
            B.cct_conv_backward_weights(t["d"], t["x"], g, t["dw"], t["db"], ws); tick(t["kind"])
            if t["gx"] is not None:
                B.cct_conv_backward_data(t["d"], t["w"], g, t["gx"], ws); tick(t["kind"])
                g = t["gx"]

    elapsed, per_step = time_steps(iteration, args.steps, args.warmup)
    ms = elapsed / args.steps * 1e3
    # shares: events after every call of one more iteration
    marks = []
    first = torch.cuda.Event(enable_timing=True)
    first.record()

    def tick(kind):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        marks.append((kind, ev))
    iteration(tick)
    torch.cuda.synchronize()
    share, prev = {}, first
    for kind, ev in marks:
        share[kind] = share.get(kind, 0.0) + prev.elapsed_time(ev)
        prev = ev
    total = sum(share.values())
    print("# CaffeNet iteration (forward + backward, every layer, no weight update), batch %d, %s: %.2f ms, %.0f images/s"
          % (N, args.precision, ms, N / ms * 1e3), file=sys.stderr)
    for k in sorted(share, key=lambda k: -share[k]):
        print("#   %-6s %7.3f ms  %5.1f %%" % (k, share[k], 100 * share[k] / total), file=sys.stderr)
    if args.per_kernel:
        prof = profiled(B, iteration, 2)
        for e in sorted(prof, key=lambda e: -e["total_ms"]):
            msk = e["total_ms"] / e["launches"]
            print("# %-44s launches/it %5.1f  avg %8.4f ms  %8.2f TFLOP/s  %8.1f GB/s" % (
                e["name"], e["launches"] / 2, msk, e["flops"] / e["launches"] / msk / 1e9,
                e["bytes"] / e["launches"] / msk / 1e6), file=sys.stderr)
    print(json.dumps({"config": "e2e", "batch": N, "precision": args.precision, "ms_per_iteration": round(ms, 3),
                      "images_per_s": round(N / ms * 1e3, 1), "gflop_per_iteration": round(flops / 1e9, 1),
                      "tflops": round(flops / 1e9 / ms, 2), "step_time_spread": spread(per_step),
                      "ms_by_kind": {k: round(v, 3) for k, v in share.items()},
                      "conv_share_of_time": round(share.get("conv", 0.0) / total, 4)}))


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (batch sharding over several GPUs is a "
                 "design note, not built); run with --gpus 1")
    import torch
    from paper_1504_04343_amd import binding as B
    from paper_1504_04343_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        B.cct_calibration_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    if args.stream_leg_only:
        types = (args.stream_leg_type,) if args.stream_leg_type else (1, 2, 3)
        prec = B.PREC_F32 if args.precision == "f32" else B.PREC_BF16_IN_F32_ACC
        print(json.dumps({"config": "materialised layouts %s, CaffeNet conv1-5, batch %d" % (
            list(types), args.batch or 256),
            "kernels": stream_kernel_leg(B, synth, args.batch or 256, prec, 2, types)}))
    elif args.config == "sweep":
        run_sweep(args, B, synth, torch)
    elif args.config == "batching":
        run_batching(args, B, synth, torch)
    elif args.config == "e2e":
        run_e2e(args, B, synth, torch)
    else:
        run_caffenet(args, B, synth, torch)


if __name__ == "__main__":
    main()
