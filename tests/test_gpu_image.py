"""GPU parity of the latent <-> image stage (the tiny autoencoder around the U-Net, appendix of the paper) and of the
step with its boundary at the u8 image, against oracle/image.py and oracle/stream.py, through the C ABI."""
import os

import numpy as np
import pytest
import torch

from workloads import CONFIGS, IMAGE_STAGE, MINI_CONFIGS, image_frames, make_weights, normal, stream_inputs

from util import TOL_BF16, TOL_BF16_MAX, check_bf16, cuda, oracle_net, rel_l2, rel_max

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4
HERE = os.path.dirname(os.path.abspath(__file__))


def _engine(wl, dtype, latent, width, n_streams=1, cfg_mode=0, timesteps=(999,), with_unet=False):
    import paper_2312_12491_amd as sd
    cfg = sd.config_from_dict(wl["unet"], latent, dtype, len(timesteps), n_streams, cfg_mode, 0, 0, width)
    eng = sd.Engine(cfg)
    if with_unet:
        eng.load_weights(make_weights(eng.manifest(), wl["seeds"]["weights"], wl["init"], dtype == "bf16"))
    blob = make_weights(eng.image_manifest(), IMAGE_STAGE["seeds"]["weights"], IMAGE_STAGE["init"], dtype == "bf16")
    eng.load_image_weights(blob)
    return eng, blob


def _oracle_params(width, bf16):
    from oracle import image as I
    return I.unpack(make_weights(I.manifest(width), IMAGE_STAGE["seeds"]["weights"], IMAGE_STAGE["init"], bf16), width)


def _u8_gap(got, want):
    d = np.abs(got.astype(np.int32) - want.astype(np.int32))
    return int(d.max()), float(d.mean()), float((d == 0).mean())


def _check_image_bf16(got, want, what):
    """Decoded float image in [0,1]: the stated relative L2 bar, and an absolute bound per pixel.  (The elementwise
    guard of the latents assumes max|o| >= 4 rms; a clamped image has max = 1 at ~2 rms, and its ReLU / clamp kinks
    give the error a heavier tail, so the guard here is absolute: 0.06 = 15 grey levels.)"""
    l2, mx = rel_l2(got, want), float(np.abs(got - want).max())
    print(f"bf16 parity {what}: rel_l2 {l2:.3e} (<= {TOL_BF16:g}), max|g-o| {mx:.3e} (<= 0.06)")
    assert l2 <= TOL_BF16 and mx <= 0.06, (what, l2, mx)


def test_image_manifest_equals_the_oracles():
    from oracle import image as I
    for dtype, width in (("fp32", 8), ("bf16", 64)):
        eng, _ = _engine(CONFIGS[1], dtype, (2, 4), width)
        assert eng.image_manifest() == [(n, tuple(s), k) for n, s, k in I.manifest(width)]
        assert eng.image_param_count() == I.param_count(width)
        eng.close()


def _roundtrip_case(dtype, width, latent, n_streams):
    """encode S seeded images, decode S seeded latents; returns per-stream (got, want) pairs."""
    from oracle import image as I
    h, w = latent
    eng, _ = _engine(CONFIGS[1], dtype, latent, width, n_streams)
    P = _oracle_params(width, dtype == "bf16")
    imgs = image_frames(IMAGE_STAGE["seeds"]["images"], 1, n_streams, 8 * h, 8 * w)[0]
    lat = torch.empty(n_streams, 4, h, w, device="cuda")
    eng.encode(cuda(imgs), lat)
    z = normal(IMAGE_STAGE["seeds"]["latents"], "latent", (n_streams, 4, h, w), 1.5)
    out_u8 = torch.empty(n_streams, 8 * h, 8 * w, 3, dtype=torch.uint8, device="cuda")
    out_f = torch.empty(n_streams, 3, 8 * h, 8 * w, device="cuda")
    eng.decode(cuda(z), out_u8, out_f)
    torch.cuda.synchronize()
    eng.close()
    res = []
    for s in range(n_streams):
        want_lat = I.encode(P, imgs[s]).numpy()
        want_img = I.decode(P, torch.as_tensor(z[s]))
        res.append((lat[s].cpu().numpy(), want_lat, out_f[s].cpu().numpy(), want_img.numpy(), out_u8[s].cpu().numpy(),
                    I.to_u8(want_img)))
    return res


@pytest.mark.parametrize("width,latent,streams", [(8, (6, 10), 2), (20, (2, 4), 1)])
def test_encode_decode_fp32(width, latent, streams):
    for glat, wlat, gimg, wimg, gu8, wu8 in _roundtrip_case("fp32", width, latent, streams):
        assert rel_max(glat, wlat) <= TOL_FP32
        assert np.abs(gimg - wimg).max() <= TOL_FP32            # the image lives in [0,1]
        mx, _, same = _u8_gap(gu8, wu8)
        assert mx <= 1 and same >= 0.995, (mx, same)             # a value within 1e-4 of a rounding boundary may flip


@pytest.mark.parametrize("width,latent,streams", [(64, (10, 18), 2), (32, (6, 10), 1), (128, (4, 6), 1)])
def test_encode_decode_bf16(width, latent, streams):
    # width 64 / 128: direct-to-LDS matrix-core kernels, ragged last row tiles at the lower resolutions; width 32: the
    # register-staged kernel
    for glat, wlat, gimg, wimg, gu8, wu8 in _roundtrip_case("bf16", width, latent, streams):
        check_bf16(glat, wlat, f"encoder width {width}")
        _check_image_bf16(gimg, wimg, f"decoder width {width}")
        mx, mean, _ = _u8_gap(gu8, wu8)
        print(f"u8 image: max level gap {mx}, mean {mean:.3f}")
        assert mx <= 12 and mean <= 1.0


def test_image_stage_at_512x512_bf16():
    path = os.path.join(HERE, "golden", "image64.npz")
    assert os.path.exists(path), f"{path} missing: run tests/golden/make_golden.py img"
    gold = np.load(path)
    st = IMAGE_STAGE
    eng, _ = _engine(CONFIGS[1], "bf16", (64, 64), st["width"])
    img = image_frames(st["seeds"]["images"], 1, 1, 512, 512)[0]
    lat = torch.empty(1, 4, 64, 64, device="cuda")
    eng.encode(cuda(img), lat)
    z = normal(st["seeds"]["latents"], "latent", (4, 64, 64), 1.5)
    out_u8 = torch.empty(1, 512, 512, 3, dtype=torch.uint8, device="cuda")
    out_f = torch.empty(1, 3, 512, 512, device="cuda")
    eng.decode(cuda(z[None]), out_u8, out_f)
    torch.cuda.synchronize()
    eng.close()
    check_bf16(lat[0].cpu().numpy(), gold["latent"], "encoder 512x512")
    _check_image_bf16(out_f[0].cpu().numpy(), gold["image_f16"].astype(np.float32), "decoder 512x512")
    mx, mean, same = _u8_gap(out_u8[0].cpu().numpy(), gold["image_u8"])
    print(f"u8 image 512x512: max level gap {mx}, mean {mean:.3f}, identical {same:.3f}")
    assert mx <= 12 and mean <= 1.0


@pytest.mark.parametrize("dtype,graph", [("fp32", True), ("fp32", False), ("bf16", True)])
def test_step_with_the_boundary_at_the_image(dtype, graph):
    # frames in, images out: encoder -> Stream Batch step (R-CFG self-negative) -> decoder against the oracle's
    # chain; the first two calls use fresh buffers (a new capture each), the rest reuse one pair (graph replay)
    from oracle import image as I
    from oracle import stream as S
    wl = MINI_CONFIGS["mini21"]           # 2 streams x 2 steps, latent 16 x 16 -> images 128 x 128
    width = 16 if dtype == "fp32" else 64
    ts, n_str = list(wl["timesteps"]), wl["n_streams"]
    h, w = wl["latent"]
    frames = 6
    eng, _ = _engine(wl, dtype, wl["latent"], width, n_str, 2, ts, with_unet=True)
    eng.use_graph(graph)
    inp = stream_inputs(wl, 1)
    eng.set_noise(inp["noise"])
    P = _oracle_params(width, dtype == "bf16")
    net = oracle_net(wl, dtype == "bf16")
    sb = S.StreamBatch(net, ts, inp["noise"], 2, 1.3, 0.8)
    imgs = image_frames(IMAGE_STAGE["seeds"]["images"] + 1, frames, n_str, 8 * h, 8 * w)
    ctx = cuda(inp["context"])
    fixed_in = torch.empty(n_str, 8 * h, 8 * w, 3, dtype=torch.uint8, device="cuda")
    fixed_out = torch.empty_like(fixed_in)
    worst, far = (0, 0.0, 1.0), 0.0
    for k in range(frames):
        if k < 2:
            fin, fout = cuda(imgs[k]), torch.empty_like(fixed_in)
        else:
            fixed_in.copy_(torch.as_tensor(imgs[k]))
            fin, fout = fixed_in, fixed_out
        valid = eng.step_image(fin, ctx, None, 1, ts, 1.3, 0.8, fout)
        torch.cuda.synchronize()
        lat = torch.stack([I.encode(P, imgs[k, s]) for s in range(n_str)])
        want_lat, wvalid = sb.step(lat, torch.as_tensor(inp["context"]), None)
        assert valid == wvalid
        if not valid:
            continue
        got = fout.cpu().numpy()
        for s in range(n_str):
            want = I.to_u8(I.decode(P, want_lat[s]))
            mx, mean, same = _u8_gap(got[s], want)
            worst = (max(worst[0], mx), max(worst[1], mean), min(worst[2], same))
            far = max(far, rel_l2(got[s], want))
    eng.close()
    print(f"{dtype} graph={graph}: u8 images, max level gap {worst[0]}, mean {worst[1]:.3f}, identical {worst[2]:.3f}, "
          f"relative L2 of the u8 image {far:.3e}")
    if dtype == "fp32":
        assert worst[0] <= 1 and worst[2] >= 0.99
    else:
        # bf16 through encoder, two U-Net evaluations per frame and decoder: the stated relative L2 bar, on the u8
        # image (plus half a grey level of quantisation, 0.3e-2 at this image's rms); single pixels next to a ReLU
        # kink can be far off, so the maximum is reported and not bounded
        assert far <= TOL_BF16 + 0.3e-2 and worst[1] <= 2.0
