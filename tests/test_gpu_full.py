"""GPU parity at the full workload sizes (SD-shaped U-Net, bf16), in the launch configuration bench.py times.

The float64 oracle needs ~10 s per U-Net row at this size, so its outputs for a prefix of each stream are
stored in tests/golden/config*.npz (written by tests/golden/make_golden.py, which calls only oracle/).  Beyond the
prefix the Stream Batch == sequential-denoising property (Sec. 3.1) is checked on sampled frames, with the
sequential side built from single-row calls of the U-Net entry point and float64 scheduler arithmetic.
"""
import os

import numpy as np
import pytest
import torch

from workloads import CONFIGS, ssf_frames, stream_inputs

from util import TOL_BF16_MAX, check_bf16, cuda, gpu_engine, rel_l2, rel_max

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2      # ||g-o|| / ||o|| on every valid output latent (and on raw eps)
TOL_SEQ = 2e-2       # stream vs sequential, both on the GPU in bf16 (different batch => different tiling / split-K)
HERE = os.path.dirname(os.path.abspath(__file__))


def _golden(c):
    path = os.path.join(HERE, "golden", f"config{c}.npz")
    assert os.path.exists(path), f"{path} missing: run tests/golden/make_golden.py {str(c).replace('_xframe', 'x')}"
    return np.load(path)


def _schedule(ts):
    betas = np.linspace(0.00085 ** 0.5, 0.012 ** 0.5, 1000, dtype=np.float64) ** 2
    al = np.cumprod(1.0 - betas)[list(ts)]
    return np.sqrt(al), np.sqrt(1.0 - al)


def _sequential_on_gpu(eng, x0, ts, noise, ctx, neg, mode, gamma, delta):
    """n single-row U-Net calls one after the other for ONE frame; x0, noise[i]: numpy [C,H,W]."""
    a, b = _schedule(ts)
    eps = torch.empty(1, *x0.shape, device="cuda")

    def unet(x, t, c):
        eng.unet_forward(cuda(x[None].astype(np.float32)), [t], c, eps)
        torch.cuda.synchronize()
        return eps[0].cpu().numpy().astype(np.float64)

    x = a[0] * x0.astype(np.float64) + b[0] * noise[0]
    ref = None
    for i, t in enumerate(ts):
        e = unet(x, t, ctx)
        if mode == 1:
            en = unet(x, t, neg)
            g = en + gamma * (e - en)
        elif mode in (2, 3):
            if i == 0:
                ref = x0.astype(np.float64) if mode == 2 else (x - b[0] * unet(x, t, neg)) / a[0]
            v = (x - a[i] * ref) / b[i]
            g = delta * v + gamma * (e - delta * v)
        else:
            g = e
        x0_hat = (x - b[i] * g) / a[i]
        if i + 1 < len(ts):
            x = a[i + 1] * x0_hat + b[i + 1] * noise[i + 1]
    return x0_hat


def _run_stream(c, mode, frames, check_seq=(), cross_frame=0):
    wl = CONFIGS[c]
    gold = _golden(f"{c}_xframe" if cross_frame else c)
    ts = list(wl["timesteps"])
    n, S = len(ts), wl["n_streams"]
    inp = stream_inputs(wl, frames)
    eng = gpu_engine(wl, "bf16", cfg_mode=mode, cross_frame=cross_frame)
    eng.set_noise(inp["noise"])
    ctx, neg = cuda(inp["context"]), cuda(inp["neg_context"])
    out = torch.empty(S, *inp["x0"].shape[2:], device="cuda")
    errs, outs = [], {}
    for k in range(frames):
        valid = eng.step(cuda(inp["x0"][k]), ctx, neg, 1, ts, wl["gamma"], wl["delta"], out)
        torch.cuda.synchronize()
        assert valid == (k >= n - 1)
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        outs[k] = got
        if k < int(gold["frames"]) and valid:
            assert bool(gold[f"mode{mode}_valid{k}"])
            errs.append(check_bf16(got[:1], gold[f"mode{mode}_frame{k}"], f"config {c} mode {mode} frame {k}")[0])
    assert len(errs) == int(gold["frames"]) - (n - 1)
    seq_errs = []
    for (f, s) in check_seq:          # frame f of stream s leaves the queue at call f + n - 1
        want = _sequential_on_gpu(eng, inp["x0"][f, s], ts, inp["noise"][:, s], ctx, neg, mode, wl["gamma"], wl["delta"])
        seq_errs.append(rel_l2(outs[f + n - 1][s], want))
    eng.close()
    return errs, seq_errs


def test_config2_single_step_sd21_shape():
    wl = CONFIGS[2]
    gold = _golden(2)
    inp = stream_inputs(wl, 2)
    eng = gpu_engine(wl, "bf16", cfg_mode=0)
    eps = torch.empty(1, 4, 64, 64, device="cuda")
    eng.unet_forward(cuda(inp["x0"][0][:1]), [999], cuda(inp["context"]), eps)
    torch.cuda.synchronize()
    check_bf16(eps.cpu().numpy(), gold["eps_row0"], "config 2 eps")
    eng.close()
    errs, _ = _run_stream(2, 0, 2)
    assert max(errs) <= TOL_BF16


def test_config3_stream_batch_of_four():
    wl = CONFIGS[3]
    gold = _golden(3)
    inp = stream_inputs(wl, 1)
    eng = gpu_engine(wl, "bf16", cfg_mode=0)
    eps = torch.empty(1, 4, 64, 64, device="cuda")
    eng.unet_forward(cuda(inp["x0"][0][:1]), [999], cuda(inp["context"]), eps)
    torch.cuda.synchronize()
    check_bf16(eps.cpu().numpy(), gold["eps_row0"], "config 3 eps")
    eng.close()
    errs, seq = _run_stream(3, 0, 40, check_seq=[(2, 0), (33, 0)])
    assert max(errs) <= TOL_BF16
    assert max(seq) <= TOL_SEQ


def _long_run(c, frames, sampled, keep_all=False):
    """The whole stated frame count through the rolling queue; Stream Batch == sequential denoising (Sec. 3.1) on
    the sampled frames, with the sequential side made of single-row U-Net calls and float64 scheduler arithmetic."""
    wl = CONFIGS[c]
    ts = list(wl["timesteps"])
    n = len(ts)
    inp = stream_inputs(wl, frames)
    eng = gpu_engine(wl, "bf16", cfg_mode=0)
    eng.set_noise(inp["noise"])
    ctx = cuda(inp["context"])
    out = torch.empty(1, *inp["x0"].shape[2:], device="cuda")
    keep = {f + n - 1 for f in sampled}
    outs, prev = {}, None
    for k in range(frames):
        valid = eng.step(cuda(inp["x0"][k]), ctx, None, 1, ts, 1.0, 1.0, out)
        assert valid == (k >= n - 1)
        if keep_all or k in keep or k % 64 == 63:
            torch.cuda.synchronize()
            got = out.cpu().numpy().copy()
            assert np.isfinite(got).all(), k
            assert prev is None or not np.array_equal(got, prev), k     # the queue moves
            prev = got
            if keep_all or k in keep:
                outs[k] = got
    torch.cuda.synchronize()
    worst = 0.0
    for f in sampled:
        want = _sequential_on_gpu(eng, inp["x0"][f, 0], ts, inp["noise"][:, 0], ctx, None, 0, 1.0, 1.0)
        l2, mx = rel_l2(outs[f + n - 1][0], want), rel_max(outs[f + n - 1][0], want)
        print(f"config {c} frame {f}: stream vs sequential rel_l2 {l2:.3e}, max|g-o|/max|o| {mx:.3e}")
        assert l2 <= TOL_SEQ and mx <= TOL_BF16_MAX, (f, l2, mx)
        worst = max(worst, l2)
    eng.close()
    return inp, outs


def test_config3_all_512_frames_through_the_queue():
    sampled = [0, 1, 63, 200, 401, 450, 499, 508]
    _long_run(3, CONFIGS[3]["frames"], sampled)


def test_config2_all_256_frames_and_the_float32_kernels():
    # n = 1: every call is a whole denoising; all 256 frames are also run on the float32 kernels of the library (a
    # second, independent opinion at full size: different kernels, no bf16 activations)
    from workloads import make_weights
    import paper_2312_12491_amd as sd
    wl = CONFIGS[2]
    sampled = [0, 31, 77, 128, 201, 230, 254, 255]
    inp, outs = _long_run(2, wl["frames"], sampled, keep_all=True)
    ts = list(wl["timesteps"])
    a, b = _schedule(ts)
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 1, 1, 0))
    eng.load_weights(make_weights(eng.manifest(), wl["seeds"]["weights"], wl["init"], True))
    eps = torch.empty(1, 4, 64, 64, device="cuda")
    ctx = cuda(inp["context"])
    worst = (0.0, 0.0)
    for f in range(wl["frames"]):
        x = a[0] * inp["x0"][f, 0].astype(np.float64) + b[0] * inp["noise"][0, 0]
        eng.unet_forward(cuda(x[None].astype(np.float32)), ts, ctx, eps)
        torch.cuda.synchronize()
        want = (x - b[0] * eps[0].cpu().numpy().astype(np.float64)) / a[0]
        l2, mx = rel_l2(outs[f][0], want), rel_max(outs[f][0], want)
        assert l2 <= TOL_BF16 and mx <= TOL_BF16_MAX, (f, l2, mx)
        worst = (max(worst[0], l2), max(worst[1], mx))
    print(f"config 2, 256 frames vs float32 kernels: worst rel_l2 {worst[0]:.3e}, worst max|g-o|/max|o| {worst[1]:.3e}")
    eng.close()


def test_config3_fp32_path_at_full_size():
    # the float32 kernels on the SD-1.5-shaped net (same bf16-rounded weights as the golden): a tight bound on the
    # full-size wiring that the bf16 tolerance cannot give
    from workloads import make_weights
    wl = CONFIGS[3]
    gold = _golden(3)
    inp = stream_inputs(wl, 1)
    import paper_2312_12491_amd as sd
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 1, 1, 0))
    eng.load_weights(make_weights(eng.manifest(), wl["seeds"]["weights"], wl["init"], True))
    eps = torch.empty(1, 4, 64, 64, device="cuda")
    eng.unet_forward(cuda(inp["x0"][0][:1]), [999], cuda(inp["context"]), eps)
    torch.cuda.synchronize()
    eng.close()
    assert rel_max(eps.cpu().numpy(), gold["eps_row0"]) <= 1e-4


def test_config3_cross_frame_attention():
    # Sec. 3.2 at full size: every level-0 self-attention runs over 4 x 4096 keys
    errs, _ = _run_stream(3, 0, 8, cross_frame=1)
    assert len(errs) == 2 and max(errs) <= TOL_BF16


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_config4_guidance_modes(mode):
    errs, seq = _run_stream(4, mode, 8, check_seq=[(3, 0)])
    assert max(errs) <= TOL_BF16
    assert max(seq) <= TOL_SEQ


def test_config5_four_streams_768():
    # (the stored oracle outputs cover stream 0: one float64 row at 96 x 96 takes the oracle about half a minute;
    # streams 1 - 3 are checked through the sequential property below, which holds per stream)
    wl = CONFIGS[5]
    errs, seq = _run_stream(5, wl["cfg_mode"], 6, check_seq=[(1, 1), (2, 2), (2, 3)])
    assert max(errs) <= TOL_BF16
    assert max(seq) <= TOL_SEQ


def test_config5_ssf_sequence_bit_exact():
    from oracle import ssf as F
    import paper_2312_12491_amd as sd
    wl = CONFIGS[1]
    spec = CONFIGS[5]["ssf"]
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 1, 1, 0))
    flt = F.Filter(spec["eta"], spec["draw_seed"])
    skips, band = 0, 0
    for k, f in enumerate(ssf_frames(spec["frame_seed"], spec["frames"], spec["h"], spec["w"])):
        want_skip, want_p = flt(f, k)
        skip, p = eng.ssf(cuda(f), spec["h"], spec["w"], spec["eta"], spec["draw_seed"], k)
        assert skip == want_skip, k
        assert p == want_p or abs(p - want_p) <= 2.3e-16 * max(p, want_p), k
        skips += skip
        band += 0.0 < p < 1.0
    assert 0 < skips < spec["frames"] and band > 0
    eng.close()


def test_hard_threshold_filter_and_run_statistics_bit_exact():
    # both filters on the 512-frame sequence: every decision equals the oracle's, hence so do duty cycle and the
    # longest stuck run; on this sequence the hard threshold processes fewer frames and stays stuck longer
    from oracle import ssf as F
    import paper_2312_12491_amd as sd
    from paper_2312_12491_amd.ssf_stats import read_statistics, run_filter
    wl = CONFIGS[1]
    spec = CONFIGS[5]["ssf"]
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 1, 1, 0))
    frames = list(ssf_frames(spec["frame_seed"], spec["frames"], spec["h"], spec["w"]))
    dev = [cuda(f) for f in frames]
    stats = {}
    for hard in (False, True):
        flt = F.Filter(spec["eta"], spec["draw_seed"], hard=hard)
        want = [flt(f, k)[0] for k, f in enumerate(frames)]
        got = run_filter(eng, dev, spec["h"], spec["w"], spec["eta"], spec["draw_seed"], hard)
        assert got == want
        stats[hard] = read_statistics(eng)      # the library's counters, against the oracle's count of its own list
        assert stats[hard] == F.run_statistics(want)
    assert stats[True]["duty_cycle"] <= stats[False]["duty_cycle"]
    assert stats[True]["longest_skip_run"] >= stats[False]["longest_skip_run"]
    eng.close()


def test_config3_runs_are_bit_identical():
    # No kernel on the path uses atomics or an order that depends on timing (split-K partials and GroupNorm partial
    # sums are folded in a fixed order), so two engines must agree bit for bit, graph replay against eager launches
    # included; a data race in a staged pipeline (an LDS buffer refilled too early) would show up here.
    wl = CONFIGS[3]
    inp = stream_inputs(wl, 8)
    ts = list(wl["timesteps"])
    ctx = cuda(inp["context"])
    runs = []
    for graph in (True, False, True):
        eng = gpu_engine(wl, "bf16", cfg_mode=0)
        eng.set_noise(inp["noise"])
        eng.use_graph(graph)
        out = torch.empty(1, 4, 64, 64, device="cuda")
        frames = []
        for k in range(8):
            eng.step(cuda(inp["x0"][k]), ctx, None, 1, ts, 1.0, 1.0, out)
            torch.cuda.synchronize()
            frames.append(out.cpu().numpy().copy())
        eng.close()
        runs.append(np.stack(frames))
    assert np.isfinite(runs[0]).all()
    assert np.array_equal(runs[0].view(np.uint32), runs[1].view(np.uint32))
    assert np.array_equal(runs[0].view(np.uint32), runs[2].view(np.uint32))
