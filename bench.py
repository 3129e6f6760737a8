"""Benchmark of the Stream Batch denoising step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: noise-in, batch assembly,
the batched U-Net at staggered timesteps, guidance, scheduler update and queue shift (sdstream_step).
Prints ONE JSON line: denoised frames/s (= streams / step time), step latency, the roofline of the dominant
kernel class (measured with HIP events around every launch in a second, profiled pass over the same steps)
and the CPU oracle timed on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def measured_traffic(config: int, mode: int, launches_per_step: float):
    """HBM bytes per launch of the implicit-GEMM class from the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE
    and WRITE_SIZE passes, scaled by what the same counters read for a plain copy).  The summary carries one line
    `bench: key=value ...` naming the workload and the launch count it was taken on; a summary of another workload,
    or of a build with a different number of launches per step (i.e. stale), gives None."""
    path = os.path.join(ROOT, "profiles", f"igemm_config{config}_hbm_traffic.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    for ln in lines:
        if ln.startswith("# bench:"):
            kv = dict(item.split("=", 1) for item in ln[len("# bench:"):].split())
            try:
                if int(kv["config"]) == config and int(kv["mode"]) == mode and \
                        abs(float(kv["launches_per_step"]) - launches_per_step) < 0.5:
                    return float(kv["traffic_bytes_per_launch"])
            except (KeyError, ValueError):
                return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload number (2..5); 3 = SD-1.5 shape, B=4, 512^2")
    ap.add_argument("--mode", type=int, default=-1, help="override cfg_mode (0 none,1 CFG,2 self,3 onetime)")
    ap.add_argument("--cross-frame", action="store_true",
                    help="Stream Batch cross-frame attention (Sec. 3.2): self-attention over the keys of all n rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--image-stage", action="store_true",
                    help="also time the step with its boundary at the u8 image (tiny autoencoder around the U-Net): "
                         "adds an `image_stage` object to the line; the headline value stays the latent-boundary step")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2312_12491_amd as sd
    from workloads import CONFIGS, IMAGE_STAGE, image_frames, make_weights, normal, stream_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    wl = CONFIGS[args.config]
    mode = wl["cfg_mode"] if args.mode < 0 else args.mode
    if isinstance(mode, tuple):
        mode = mode[1]
    ts = list(wl["timesteps"])
    n, S = len(ts), wl["n_streams"]
    cfg = sd.config_from_dict(wl["unet"], wl["latent"], wl["dtype"], n, S, mode, 0, int(args.cross_frame))
    eng = sd.Engine(cfg)
    blob = make_weights(eng.manifest(), wl["seeds"]["weights"], wl["init"], wl["dtype"] == "bf16")
    eng.load_weights(blob)
    inp = stream_inputs(wl, 8)
    eng.set_noise(inp["noise"])
    eng.use_graph(not args.no_graph)
    x0 = [torch.as_tensor(inp["x0"][k]).cuda() for k in range(8)]
    ctx = torch.as_tensor(inp["context"]).cuda()
    neg = torch.as_tensor(inp["neg_context"]).cuda()
    out = torch.empty_like(x0[0])
    gamma, delta = float(wl["gamma"]), float(wl["delta"])

    def step(k):
        eng.step(x0[k % 8], ctx, neg, 1, ts, gamma, delta, out)

    if args.calib_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    fps = S * args.steps / dt
    assert torch.isfinite(out).all() or os.environ.get("SDSTREAM_EXP")   # (timing experiments of development builds leave garbage)

    rows = eng.max_batch()
    step_flops = eng.flops_per_row() * rows
    util = step_flops / (ms_per_step * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)

    # second pass, kernel by kernel with HIP events on the same stream, for the per-class roofline
    eng.profile_enable(True)
    eng.profile_reset()
    for k in range(args.profile_steps):
        step(k)
    prof = eng.profile_read()
    eng.profile_enable(False)
    classes = {}
    for name, r in prof.items():
        classes[name] = dict(launches_per_step=r["launches"] / args.profile_steps,
                             ms_per_step=r["ms"] / args.profile_steps,
                             tflops=r["flops"] / (r["ms"] * 1e-3) / 1e12 if r["ms"] > 0 else 0.0,
                             gbs=r["bytes"] / (r["ms"] * 1e-3) / 1e9 if r["ms"] > 0 else 0.0)
    for name, c in classes.items():   # fraction of the roofline that bounds the class (event time, dispatch gap included)
        c["frac_of_peak"] = c["tflops"] / PEAK_BF16_TFLOPS if name.endswith("mfma") else c["gbs"] / PEAK_HBM_GBS
        c["bound"] = "mfma" if name.endswith("mfma") else "hbm"
    # An event pair around an eager launch also spans a dispatch gap.  The same kernels replayed as a graph take
    # ms_per_step in total, so the gap per bracketed launch is what makes the bracketed times add up to that.
    n_pairs = sum(c["launches_per_step"] for c in classes.values())
    pair_us = max(0.0, (sum(c["ms_per_step"] for c in classes.values()) - ms_per_step) * 1e3 / n_pairs)
    dom = max((c for c in classes if c.startswith("igemm")), key=lambda c: classes[c]["ms_per_step"])
    peak = PEAK_BF16_TFLOPS if dom.endswith("mfma") else PEAK_FP32_TFLOPS
    dr = prof[dom]
    launch_us = dr["ms"] * 1e3 / dr["launches"] - pair_us
    achieved = dr["flops"] / dr["launches"] / (launch_us * 1e-6) / 1e12
    # HBM-side bytes per launch of this kernel class, from the two rocprofv3 --pmc passes summarised under profiles/
    # (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a 256 MiB copy); only valid for the workload they were taken on
    traffic = measured_traffic(args.config, mode, dr["launches"] / args.profile_steps) \
        if dom == "igemm_mfma" and not args.cross_frame else None
    roofline = {"kernel": dom, "bound": "mfma" if dom.endswith("mfma") else "alu",
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "avg_launch_us": launch_us, "event_pair_overhead_us": pair_us,
                "launches_per_step": dr["launches"] / args.profile_steps,
                "algorithmic_bytes_per_launch": dr["bytes"] / dr["launches"], "traffic": traffic}

    # what a kernel of nothing but register-fed bf16 MFMAs reaches on this device right now (clock actually held)
    mfma_ceiling = eng.mfma_ceiling(20000)

    cpu_baseline = None
    if not args.no_cpu_baseline and not args.cross_frame:   # (a cross-frame batch has no one-row sample)
        from oracle import unet as U
        shape = U.UNetShape.from_dict(wl["unet"])
        net = U.UNet(shape, blob)
        xs = torch.as_tensor(inp["x0"][0][:1])
        t1 = time.perf_counter()
        net(xs, [ts[0]], torch.as_tensor(inp["context"]))
        t_row = time.perf_counter() - t1
        cpu_baseline = {"value": 1.0 / (t_row * rows / S), "unit": "frames/s", "cores": min(torch.get_num_threads(), len(os.sched_getaffinity(0))),
                        "kind": "oracle", "sample": f"one U-Net row of the {rows}-row step (float64), "
                        f"{t_row:.1f} s, scaled to {rows} rows; the elementwise tail is negligible"}

    image_stage = None
    if args.image_stage:
        eng.close()
        icfg = sd.config_from_dict(wl["unet"], wl["latent"], wl["dtype"], n, S, mode, 0, int(args.cross_frame),
                                   IMAGE_STAGE["width"])
        eng = sd.Engine(icfg)
        eng.load_weights(blob)
        eng.load_image_weights(make_weights(eng.image_manifest(), IMAGE_STAGE["seeds"]["weights"], IMAGE_STAGE["init"],
                                            wl["dtype"] == "bf16"))
        eng.set_noise(inp["noise"])
        H, W = 8 * wl["latent"][0], 8 * wl["latent"][1]
        frames = torch.as_tensor(image_frames(IMAGE_STAGE["seeds"]["images"], 2, S, H, W)).cuda()
        img_out = torch.empty_like(frames[0])
        lat = torch.empty(S, 4, *wl["latent"], device="cuda")

        def timed(fn, reps):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / reps * 1e3
        ms_img_step = timed(lambda: eng.step_image(frames[0], ctx, neg, 1, ts, gamma, delta, img_out), args.steps)
        ms_enc = timed(lambda: eng.encode(frames[0], lat), args.steps)
        ms_dec = timed(lambda: eng.decode(lat, img_out, None), args.steps)
        gf = 1e-9 * S * H * W * (2 * 27 * 64 + 2 * 64 * 27)   # first / last convolutions
        per_px = 2.0 * 9 * 64 * 64                            # one 64 -> 64 convolution per output pixel
        px = [H * W / 4 ** k for k in range(4)]
        enc_gf = 1e-9 * S * per_px * (3 * px[0] + 10 * (px[1] + px[2] + px[3])) + 1e-9 * S * px[3] * 2 * 9 * 64 * 4
        dec_gf = 1e-9 * S * per_px * (9 * px[3] + 10 * (px[2] + px[1]) + 4 * px[0]) + 1e-9 * S * px[3] * 2 * 9 * 64 * 4
        image_stage = {"workload": f"{S} image(s) {H}x{W}x3 u8 per step, autoencoder width {IMAGE_STAGE['width']}",
                       "step_image_ms": ms_img_step, "frames_per_s": S / (ms_img_step * 1e-3),
                       "encode_ms": ms_enc, "decode_ms": ms_dec,
                       "encode_tflops": (enc_gf + gf / 2) / ms_enc, "decode_tflops": (dec_gf + gf / 2) / ms_dec}

    line = {
        "metric": "denoised frames/sec (Stream Batch step)", "value": fps, "unit": "frames/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl["dtype"], "data": "synthetic",
        "config": {"workload": f"config {args.config}: {wl['name']}, latent {wl['latent'][0]}x{wl['latent'][1]}, "
                               f"n={n} steps x S={S} streams, cfg_mode={mode}, U-Net batch {rows}"
                               + (", cross-frame attention" if args.cross_frame else ""),
                   "timesteps": ts, "graph": not args.no_graph},
        "unet_step_ms": ms_per_step, "step_tflop": step_flops / 1e12, "mfma_util": util,
        "peak_assumed_tflops": PEAK_BF16_TFLOPS, "mfma_only_kernel_tflops": mfma_ceiling,
        "roofline": roofline, "kernel_classes": classes, "cpu_baseline": cpu_baseline,
        "image_stage": image_stage,
        "context": "paper: 91.07 fps whole pipeline on one RTX 4090 (other hardware, includes VAE): not a target",
    }
    print(json.dumps(line))
    eng.close()


if __name__ == "__main__":
    main()
