#!/usr/bin/env python3
"""Benchmark of the lowering-based convolutional layer on one MI355X.

One "step" = the whole hot path over one batch: forward, backward-data and
backward-weights of CaffeNet conv1..conv5 at batch 256 (15 passes; lowering, multiply and
lifting all inside the timed region; inputs, weights, upstream gradients and the workspace
already resident in HBM).  Prints ONE JSON line with the headline metric (algorithmic conv
GFLOP/s), the roofline figures of the dominant kernel (measured with HIP events on the
launching stream) and the CPU oracle's rate on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_caffenet_b256_f32.txt")


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (None if absent)."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.rstrip("\n").split("\t")
            if not line.startswith("#") and len(f) >= 2 and f[0] == kernel:
                return int(f[1])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--precision", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--lowering", type=int, default=0, help="0 = auto (default), 1..3 = force")
    ap.add_argument("--chunk", type=int, default=0, help="images per chunk (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-images", type=int, default=64)
    ap.add_argument("--per-kernel", action="store_true", help="also print the per-kernel table")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain 1 GiB device copy (reference row for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE scaling)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (batch sharding over several GPUs is a "
                 "design note, not built); run with --gpus 1")
    import numpy as np
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
    prec = B.PREC_F32 if args.precision == "f32" else B.PREC_BF16_IN_F32_ACC
    layers = synth.caffenet(args.batch)
    passes = [B.PASS_FORWARD, B.PASS_BACKWARD_DATA, B.PASS_BACKWARD_WEIGHTS]

    # ---- resident inputs -------------------------------------------------------------------
    state = []
    ws_bytes = 0
    for L in layers:
        d = B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, args.lowering, prec)
        t = dict(L=L, d=d,
                 x=torch.from_numpy(synth.make_x(L)).cuda(), w=torch.from_numpy(synth.make_w(L)).cuda(),
                 b=torch.from_numpy(synth.make_bias(L)).cuda(), dy=torch.from_numpy(synth.make_dy(L)).cuda())
        t["y"] = torch.empty_like(t["dy"])
        t["dx"] = torch.empty_like(t["x"])
        t["dw"] = torch.empty_like(t["w"])
        t["db"] = torch.empty_like(t["b"])
        t["picked"] = {p: (args.lowering or B.cct_pick_lowering(d, p)) for p in passes}
        for p in passes:
            n = B.cct_conv_workspace_bytes(d, p) if not args.chunk else \
                B.cct_conv_workspace_bytes_for_chunk(d, p, min(args.chunk, L.N))
            ws_bytes = max(ws_bytes, n)
        state.append(t)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flops_per_step = sum(L.flops for L in layers) * len(passes)

    def step():
        for t in state:
            d = t["d"]
            B.cct_conv_forward(d, t["x"], t["w"], t["b"], t["y"], ws)
            B.cct_conv_backward_data(d, t["w"], t["dy"], t["dx"], ws)
            if B.PASS_BACKWARD_WEIGHTS in passes:
                B.cct_conv_backward_weights(d, t["x"], t["dy"], t["dw"], t["db"], ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    gflops = flops_per_step / 1e9 / (elapsed / args.steps)

    # ---- per-kernel HIP-event timing over the same steps (second leg, same launches) --------
    B.cct_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    B.cct_profile_enable(False)
    prof = B.cct_profile_read(64)
    total_kernel_ms = sum(e["total_ms"] for e in prof)
    def is_mfma(e):   # the GEMMs and the fused conv kernel (matrix-core bound); the rest stream
        return e["name"].startswith(("gemm_", "conv_fused", "conv_bwdw_fused"))
    gemms = [e for e in prof if is_mfma(e)]
    dom = max(gemms, key=lambda e: e["total_ms"])
    avg_ms = dom["total_ms"] / dom["launches"]
    achieved_tflops = dom["flops"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
    peak = PEAK_FP32_MFMA_TFLOPS if args.precision == "f32" else PEAK_BF16_MFMA_TFLOPS
    roofline = {
        "bound": "mfma", "kernel": dom["name"], "achieved": round(achieved_tflops, 2), "peak": peak,
        "unit": "TFLOP/s", "frac": round(achieved_tflops / peak, 4),
        "traffic": measured_traffic(dom["name"]) if (args.precision == "f32" and args.batch == 256 and
                                                     not args.lowering and not args.chunk) else None,
        "algorithmic_bytes_per_launch": int(dom["bytes"] / dom["launches"]),
        "avg_launch_ms": round(avg_ms, 4), "launches_per_step": dom["launches"] / args.steps,
        "share_of_step_kernel_time": round(dom["total_ms"] / total_kernel_ms, 3),
    }
    all_gemm_flops = sum(e["flops"] for e in gemms)
    all_gemm_ms = sum(e["total_ms"] for e in gemms)
    # the lowering / lifting kernels proper (pack, split-K reduce and dbias are small helpers)
    streams = [e for e in prof if e["name"].startswith(("lower_", "lift_", "inv_lift_", "inv_lower_"))]
    stream_bytes = sum(e["bytes"] for e in streams)
    stream_ms = sum(e["total_ms"] for e in streams)
    phases = {
        "all_gemm_tflops": round(all_gemm_flops / (all_gemm_ms * 1e-3) / 1e12, 2),
        "all_gemm_frac_of_%s_mfma_peak" % ("fp32" if args.precision == "f32" else "bf16"):
            round(all_gemm_flops / (all_gemm_ms * 1e-3) / 1e12 / peak, 4),
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

    # ---- CPU oracle on a bounded sample of the same workload --------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_images, args.batch)
        cpu_flops, cpu_s = 0.0, 0.0
        for t in state:
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

    out = {
        "metric": "conv GFLOP/s fwd+bwd, CaffeNet conv1-5 batch 256; % fp32 MFMA peak",
        "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.precision == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": "CaffeNet conv1-5 forward + backward-data + backward-weights, batch %d, "
                               "fp32, auto lowering" % args.batch if args.precision == "f32" and not args.lowering
                   else "CaffeNet conv1-5, batch %d, precision %s, lowering %d, passes %d" % (
                       args.batch, args.precision, args.lowering, len(passes)),
                   "batch": args.batch, "gflop_per_step": round(flops_per_step / 1e9, 2),
                   "lowering_picked": {t["L"].name: [t["picked"][p] for p in passes] for t in state},
                   "workspace_MiB": ws_bytes >> 20,
                   "frac_of_%s_mfma_peak" % ("fp32" if args.precision == "f32" else "bf16"):
                       round(gflops / 1e3 / (PEAK_FP32_MFMA_TFLOPS if args.precision == "f32"
                                             else PEAK_BF16_MFMA_TFLOPS), 4)},
        "roofline": roofline,
        "phases": phases,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
