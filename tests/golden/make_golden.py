"""Writes the oracle's expected outputs for the full-size (SD-shaped) workloads into tests/golden/*.npz.

Calls only oracle/ and the seeded generators in workloads/ (never the HIP library).  The SD-shaped U-Net
costs the float64 oracle ~10 s per row on 8 cores, so these prefixes are computed once here and the GPU
tests compare against the stored arrays:
  config 2: first 2 frames;  config 3: first 6 frames (3 valid outputs);  config 4: first 6 frames in each of
  the three guidance modes;  config 5: first 5 frames of stream 0 (2 valid outputs);  plus one raw eps row
  (t = 999) per U-Net shape;  "3x": config 3 with Stream Batch cross-frame attention (Sec. 3.2), first 5 frames
  (2 valid outputs), into config3_xframe.npz.
  "img": the latent <-> image stage at width 64 and 512 x 512: the latent of one seeded image and the image of one
  seeded latent (float16 copy of the float image plus the u8 image), into image64.npz.
Usage: python tests/golden/make_golden.py [config ...]
"""
import os
import sys
import time

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import stream as S  # noqa: E402
from oracle import unet as U  # noqa: E402
from workloads import CONFIGS, make_weights, stream_inputs  # noqa: E402

FRAMES = {2: 2, 3: 6, 4: 6, 5: 5}


def run(c: int, cross_frame: bool = False):
    wl = CONFIGS[c]
    shape = U.UNetShape.from_dict(wl["unet"])
    t0 = time.time()
    net = U.UNet(shape, make_weights(U.manifest(shape), wl["seeds"]["weights"], wl["init"], wl["dtype"] == "bf16"),
                 cross_frame=cross_frame)
    frames = 5 if cross_frame else FRAMES[c]
    inp = stream_inputs(wl, frames)
    ctx, neg = torch.as_tensor(inp["context"]), torch.as_tensor(inp["neg_context"])
    ts = list(wl["timesteps"])
    modes = wl["cfg_mode"] if isinstance(wl["cfg_mode"], tuple) else (wl["cfg_mode"],)
    out = {"frames": np.int64(frames)}
    eps = net(torch.as_tensor(inp["x0"][0][:1]), [ts[0]], ctx)
    out["eps_row0"] = eps.numpy().astype(np.float32)
    for mode in modes:
        sb = S.StreamBatch(net, ts, inp["noise"][:, :1], mode, wl["gamma"], wl["delta"])
        for k in range(frames):
            o, valid = sb.step(inp["x0"][k][:1], ctx, neg)
            out[f"mode{mode}_frame{k}"] = o.numpy().astype(np.float32)
            out[f"mode{mode}_valid{k}"] = np.bool_(valid)
            print(f"config {c} mode {mode} frame {k} valid={valid} ({time.time() - t0:.0f} s)", flush=True)
    np.savez_compressed(os.path.join(HERE, f"config{c}_xframe.npz" if cross_frame else f"config{c}.npz"), **out)


def run_image():
    from oracle import image as I
    from workloads import IMAGE_STAGE, image_frames, normal
    st = IMAGE_STAGE
    t0 = time.time()
    P = I.unpack(make_weights(I.manifest(st["width"]), st["seeds"]["weights"], st["init"], True), st["width"])
    img = image_frames(st["seeds"]["images"], 1, 1, 512, 512)[0, 0]
    lat = I.encode(P, img)
    print(f"image stage: encoded ({time.time() - t0:.0f} s)", flush=True)
    z = normal(st["seeds"]["latents"], "latent", (4, 64, 64), 1.5)
    dec = I.decode(P, torch.as_tensor(z))
    print(f"image stage: decoded ({time.time() - t0:.0f} s)", flush=True)
    np.savez_compressed(os.path.join(HERE, "image64.npz"), latent=lat.numpy().astype(np.float32),
                        image_f16=dec.numpy().astype(np.float16), image_u8=I.to_u8(dec))


if __name__ == "__main__":
    for a in (sys.argv[1:] or ["2", "3", "4", "5", "3x", "img"]):
        if a == "img":
            run_image()
        else:
            run(int(a.rstrip("x")), a.endswith("x"))
