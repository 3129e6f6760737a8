"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, MINI_CONFIGS, normal, ssf_frames, stream_inputs

from util import TOL_BF16_MAX, check_bf16, cuda, gpu_engine, oracle_net, rel_l2, rel_max

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4   # max|g-o| / max|o|
TOL_BF16 = 2e-2   # ||g-o|| / ||o||


def _unet_case(wl, dtype, rows, ts):
    import oracle.unet  # noqa: F401
    net = oracle_net(wl, dtype == "bf16")
    eng = gpu_engine(wl, dtype, cfg_mode=1, n_streams=1, timesteps=list(range(len(ts), 0, -1)))
    u = wl["unet"]
    h, w = wl["latent"]
    x = normal(wl["seeds"]["inputs"], "unet_x", (rows, u["in_channels"], h, w))
    ctx = normal(wl["seeds"]["context"], "context", (u["context_len"], u["context_dim"]))
    assert rows <= eng.max_batch()
    out = torch.empty(rows, u["in_channels"], h, w, device="cuda")
    eng.unet_forward(cuda(x), ts, cuda(ctx), out)
    torch.cuda.synchronize()
    want = net(torch.as_tensor(x), ts, torch.as_tensor(ctx)).numpy()
    eng.close()
    return out.cpu().numpy(), want


def test_manifest_equals_the_oracles():
    from oracle import unet as U
    for wl in [CONFIGS[1], CONFIGS[3], MINI_CONFIGS["mini40"]]:
        for dtype in ("fp32", "bf16"):
            import paper_2312_12491_amd as sd
            eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], dtype, 1, 1, 0))
            shape = U.UNetShape.from_dict(wl["unet"])
            assert eng.manifest() == [(n, tuple(s), k) for n, s, k in U.manifest(shape)]
            assert eng.param_count() == U.param_count(shape)
            eng.close()


def test_unet_tiny_fp32():
    got, want = _unet_case(CONFIGS[1], "fp32", 3, [999, 499, 7])
    assert rel_max(got, want) <= TOL_FP32


@pytest.mark.parametrize("name", ["mini15", "mini21", "mini40"])
def test_unet_mini_fp32(name):
    got, want = _unet_case(MINI_CONFIGS[name], "fp32", 2, [999, 259])
    assert rel_max(got, want) <= TOL_FP32


@pytest.mark.parametrize("name", ["mini15", "mini21", "mini40"])
def test_unet_mini_bf16(name):
    got, want = _unet_case(MINI_CONFIGS[name], "bf16", 2, [999, 259])
    check_bf16(got, want, name)


def test_unet_wide_first_level_with_a_ragged_row_tile_bf16():
    # 4 rows x 62 x 58 pixels x 320 channels: the row-resident GEMM kernels of the 1x1 layers, last row tile ragged
    got, want = _unet_case(MINI_CONFIGS["wide320"], "bf16", 4, [999, 759, 499, 259])
    check_bf16(got, want, "wide320")


def test_stream_wide_first_level_full_cfg_bf16():
    # two prompts on 2 + 2 rows of 3596 pixels: the boundary between them falls inside a row tile, so the folded
    # cross-attention runs as two launches on row ranges, each with the kernel chosen for the whole range
    wl = MINI_CONFIGS["wide320"]
    worst_max, worst = _stream_case(wl, "bf16", 1, 1.2, 1.0, 3)
    print(f"wide320 full CFG: rel_l2 {worst:.3e}, max|g-o|/max|o| {worst_max:.3e}")
    assert worst <= TOL_BF16
    assert worst_max <= TOL_BF16_MAX


@pytest.mark.parametrize("name,dtype", [("mini15", "fp32"), ("mini40", "fp32"), ("mini15", "bf16"), ("mini21", "bf16"),
                                        ("mini40", "bf16")])
def test_unet_mini_with_random_norm_scales_and_shifts(name, dtype):
    # the workloads' norms have scale 1 and shift 0; here every GroupNorm and LayerNorm has random ones, so a scale
    # or shift that a kernel drops, misplaces or folds into the wrong matrix shows
    wl = dict(MINI_CONFIGS[name], init="fanin_affine")
    got, want = _unet_case(wl, dtype, 3, [999, 499, 20])
    if dtype == "fp32":
        assert rel_max(got, want) <= TOL_FP32
    else:
        check_bf16(got, want, name + " affine norms")


def _stream_case(wl, dtype, mode, gamma, delta, frames, sched=0, graph=True, swap_prompt_at=None):
    """swap_prompt_at = k: from call k on the positive and the negative prompt change places (a new context_epoch)."""
    from oracle import stream as S
    net = oracle_net(wl, dtype == "bf16")
    inp = stream_inputs(wl, frames)
    ts = list(wl["timesteps"])
    sb = S.StreamBatch(net, ts, inp["noise"], mode, gamma, delta, ("lcm", "ddim", "lcm_exact")[sched])
    ctx, neg = torch.as_tensor(inp["context"]), torch.as_tensor(inp["neg_context"])
    eng = gpu_engine(wl, dtype, cfg_mode=mode, scheduler=sched)
    eng.use_graph(graph)
    eng.set_noise(inp["noise"])
    dctx, dneg = cuda(inp["context"]), cuda(inp["neg_context"])
    out = torch.empty_like(cuda(inp["x0"][0]))
    worst_max, worst_l2, n_valid = 0.0, 0.0, 0
    for k in range(frames):
        epoch = 1
        if swap_prompt_at is not None and k == swap_prompt_at:
            ctx, neg, dctx, dneg = neg, ctx, dneg, dctx
        if swap_prompt_at is not None and k >= swap_prompt_at:
            epoch = 2
        valid = eng.step(cuda(inp["x0"][k]), dctx, dneg, epoch, ts, gamma, delta, out)
        torch.cuda.synchronize()
        want, wvalid = sb.step(inp["x0"][k], ctx, neg)
        assert valid == wvalid
        if valid:
            n_valid += 1
            worst_max = max(worst_max, rel_max(out.cpu().numpy(), want.numpy()))
            worst_l2 = max(worst_l2, rel_l2(out.cpu().numpy(), want.numpy()))
    eng.close()
    assert n_valid == frames - (len(ts) - 1)
    return worst_max, worst_l2


def test_config1_stream_all_frames():
    wl = CONFIGS[1]
    worst, _ = _stream_case(wl, "fp32", wl["cfg_mode"], wl["gamma"], wl["delta"], wl["frames"])
    assert worst <= TOL_FP32


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("sched", [0, 1])
def test_stream_modes_mini_fp32(mode, sched):
    wl = MINI_CONFIGS["mini21"]       # 2 streams x 2 steps
    worst, _ = _stream_case(wl, "fp32", mode, 1.3, 0.8, 4, sched, graph=(mode % 2 == 0))
    assert worst <= TOL_FP32


@pytest.mark.parametrize("mode", [0, 2])
def test_exact_consistency_parameterisation_fp32(mode):
    # scheduler 2 (c_skip, c_out of the appendix) at timesteps small enough for them to differ from (0, 1):
    # c_skip(2) = 6.2e-4, and the last slot at tau = 0 is the boundary condition x0 = x
    wl = dict(MINI_CONFIGS["mini21"], timesteps=(2, 0))
    worst, _ = _stream_case(wl, "fp32", mode, 1.3, 0.8, 4, 2)
    assert worst <= TOL_FP32
    wl = dict(MINI_CONFIGS["mini21"])
    worst, _ = _stream_case(wl, "fp32", mode, 1.3, 0.8, 3, 2, graph=False)
    assert worst <= TOL_FP32


@pytest.mark.parametrize("mode", [1, 3])
def test_prompt_change_while_the_queue_is_live_fp32(mode):
    # the prompt's cached keys / values are rebuilt when context_epoch changes; frames already in the queue go on
    wl = MINI_CONFIGS["mini15"]       # 1 stream x 4 steps
    worst, _ = _stream_case(wl, "fp32", mode, 1.3, 0.8, 9, swap_prompt_at=5)
    assert worst <= TOL_FP32


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_stream_modes_mini_bf16(mode):
    wl = MINI_CONFIGS["mini15"]       # 1 stream x 4 steps
    worst_max, worst = _stream_case(wl, "bf16", mode, 1.2, 1.0, 6)
    print(f"mode {mode}: rel_l2 {worst:.3e}, max|g-o|/max|o| {worst_max:.3e}")
    assert worst <= TOL_BF16
    assert worst_max <= TOL_BF16_MAX


def test_set_noise_on_a_used_engine_starts_from_an_empty_queue_fp32():
    # cross-frame attention lets the not-yet-valid rows take part, so leftovers of an earlier run in the queue would
    # change the first outputs after set_noise; the oracle's queue starts at zero
    from oracle import stream as S
    wl = MINI_CONFIGS["mini15"]
    ts = list(wl["timesteps"])
    eng = gpu_engine(wl, "fp32", cfg_mode=2, cross_frame=1)
    dctx = None
    for run in range(2):
        inp = stream_inputs(dict(wl, seeds=dict(wl["seeds"], noise=wl["seeds"]["noise"] + run,
                                                inputs=wl["seeds"]["inputs"] + run)), 6)
        eng.set_noise(inp["noise"])
        dctx = cuda(inp["context"])
        out = torch.empty_like(cuda(inp["x0"][0]))
        net = oracle_net(wl, False, cross_frame=True)
        sb = S.StreamBatch(net, ts, inp["noise"], 2, 1.3, 0.8)
        for k in range(6):
            valid = eng.step(cuda(inp["x0"][k]), dctx, None, 1, ts, 1.3, 0.8, out)
            torch.cuda.synchronize()
            want, wvalid = sb.step(inp["x0"][k], torch.as_tensor(inp["context"]), None)
            assert valid == wvalid
            if valid:
                assert rel_max(out.cpu().numpy(), want.numpy()) <= TOL_FP32, (run, k)
    eng.close()


def test_ssf_decisions_bit_exact():
    from oracle import ssf as F
    import paper_2312_12491_amd as sd
    wl = CONFIGS[1]
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 1, 1, 0))
    for (h, w, n, eta) in [(48, 64, 80, 0.98), (37, 21, 45, 0.9), (512, 512, 24, 0.98), (48, 64, 30, 1.0)]:
        eng.reset()
        flt = F.Filter(eta, 7000)
        kinds = set()
        for k, f in enumerate(ssf_frames(6000, n, h, w)):
            want_skip, want_p = flt(f, k)
            skip, p = eng.ssf(cuda(f), h, w, eta, 7000, k)
            assert skip == want_skip, (h, w, k)
            assert p == want_p or abs(p - want_p) <= 2.3e-16 * max(p, want_p)
            kinds.add(skip)
        assert eta >= 1.0 or kinds == {True, False}
        assert eta < 1.0 or kinds == {False}
    eng.close()


def test_error_paths_leave_the_engine_usable():
    import paper_2312_12491_amd as sd
    wl = CONFIGS[1]
    u = wl["unet"]
    bad = sd.config_from_dict(dict(u, num_heads=2), wl["latent"], "fp32", 2, 1, 0)   # both head fields set
    with pytest.raises(sd.SdstreamError) as ei:
        sd.Engine(bad)
    assert ei.value.code == -1
    eng = sd.Engine(sd.config_from_dict(u, wl["latent"], "fp32", 2, 1, 3))
    inp = stream_inputs(wl, 1)
    x, ctx = cuda(inp["x0"][0]), cuda(inp["context"])
    out = torch.empty_like(x)
    with pytest.raises(sd.SdstreamError) as ei:
        eng.step(x, ctx, ctx, 1, [999, 499], 1.0, 1.0, out)
    assert ei.value.code == -2                                                        # weights not loaded
    from workloads import make_weights
    blob = make_weights(eng.manifest(), 1, "n002", False)
    with pytest.raises(sd.SdstreamError) as ei:
        eng._check(eng._l.sdstream_load_weights(eng._h, blob.ctypes.data, blob.nbytes - 4))
    assert ei.value.code == -3
    eng.load_weights(blob)
    with pytest.raises(sd.SdstreamError) as ei:
        eng.step(x, ctx, ctx, 1, [999, 499], 1.0, 1.0, out)
    assert ei.value.code == -2                                                        # noise cache not set
    eng.set_noise(inp["noise"])
    for ts in ([499, 999], [999, 999], [1000, 5], [999, -1]):
        with pytest.raises(sd.SdstreamError) as ei:
            eng.step(x, ctx, ctx, 1, ts, 1.0, 1.0, out)
        assert ei.value.code == -1
    with pytest.raises(sd.SdstreamError) as ei:
        eng.step(x, ctx, None, 1, [999, 499], 1.0, 1.0, out)                          # onetime needs neg_context
    assert ei.value.code == -1
    assert eng.step(x, ctx, ctx, 1, [999, 499], 1.0, 1.0, out) is False
    assert eng.step(x, ctx, ctx, 1, [999, 499], 1.0, 1.0, out) is True
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    eng.close()


def test_mfma_ceiling_probe_reports_a_plausible_rate():
    # the register-only MFMA kernel cannot beat the published dense bf16 peak and should get well past half of it
    import paper_2312_12491_amd as sd
    wl = CONFIGS[1]
    eng = sd.Engine(sd.config_from_dict(wl["unet"], wl["latent"], "fp32", 2, 1, 0))
    rate = eng.mfma_ceiling(20000)
    assert 1500.0 < rate < 2600.0, rate
    for iters in (0, -3, (1 << 20) + 1):
        with pytest.raises(sd.SdstreamError) as ei:
            eng.mfma_ceiling(iters)
        assert ei.value.code == -1
    eng.close()
