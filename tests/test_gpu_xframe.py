"""GPU parity of Stream Batch cross-frame attention (Sec. 3.2 of the paper) against the oracle: the U-Net on whole
stream batches, the full step in every guidance mode, and the cases that must not notice the option."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, MINI_CONFIGS, normal, stream_inputs

from util import TOL_BF16_MAX, check_bf16, cuda, gpu_engine, oracle_net, rel_l2, rel_max

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4   # max|g-o| / max|o|
TOL_BF16 = 2e-2   # ||g-o|| / ||o||


def _unet_groups(wl, dtype, n, groups, extra):
    """U-Net forward on `groups` stream batches of n rows plus `extra` rows that stay alone."""
    net = oracle_net(wl, dtype == "bf16", cross_frame=True)
    rows = n * groups + extra
    eng = gpu_engine(wl, dtype, cfg_mode=1, n_streams=(rows + 2 * n - 1) // (2 * n), timesteps=list(range(n, 0, -1)),
                     cross_frame=1)
    assert rows <= eng.max_batch()
    u = wl["unet"]
    h, w = wl["latent"]
    x = normal(wl["seeds"]["inputs"], "unet_x", (rows, u["in_channels"], h, w))
    ctx = normal(wl["seeds"]["context"], "context", (u["context_len"], u["context_dim"]))
    ts = [999 - 173 * r for r in range(rows)]
    out = torch.empty(rows, u["in_channels"], h, w, device="cuda")
    eng.unet_forward(cuda(x), ts, cuda(ctx), out)
    torch.cuda.synchronize()
    eng.close()
    want = []
    for g in range(groups):
        sl = slice(g * n, (g + 1) * n)
        want.append(net(torch.as_tensor(x[sl]), ts[sl], torch.as_tensor(ctx)))
    for r in range(n * groups, rows):
        want.append(net(torch.as_tensor(x[r:r + 1]), ts[r:r + 1], torch.as_tensor(ctx)))
    return out.cpu().numpy(), torch.cat(want).numpy()


@pytest.mark.parametrize("name,n,groups,extra", [("mini15", 3, 1, 0), ("mini21", 2, 2, 1), ("mini40", 2, 1, 1)])
def test_unet_batches_fp32(name, n, groups, extra):
    got, want = _unet_groups(MINI_CONFIGS[name], "fp32", n, groups, extra)
    assert rel_max(got, want) <= TOL_FP32


@pytest.mark.parametrize("name,n,groups,extra", [("mini15", 4, 1, 0), ("mini40", 2, 2, 1)])
def test_unet_batches_bf16(name, n, groups, extra):
    got, want = _unet_groups(MINI_CONFIGS[name], "bf16", n, groups, extra)
    check_bf16(got, want, name + " cross-frame")


def _stream_case(wl, dtype, mode, gamma, delta, frames, graph=True):
    from oracle import stream as S
    net = oracle_net(wl, dtype == "bf16", cross_frame=True)
    inp = stream_inputs(wl, frames)
    ts = list(wl["timesteps"])
    sb = S.StreamBatch(net, ts, inp["noise"], mode, gamma, delta)
    ctx, neg = torch.as_tensor(inp["context"]), torch.as_tensor(inp["neg_context"])
    eng = gpu_engine(wl, dtype, cfg_mode=mode, cross_frame=1)
    eng.use_graph(graph)
    eng.set_noise(inp["noise"])
    dctx, dneg = cuda(inp["context"]), cuda(inp["neg_context"])
    out = torch.empty_like(cuda(inp["x0"][0]))
    worst_max, worst_l2, n_valid = 0.0, 0.0, 0
    for k in range(frames):
        valid = eng.step(cuda(inp["x0"][k]), dctx, dneg, 1, ts, gamma, delta, out)
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


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_stream_modes_fp32(mode):
    wl = MINI_CONFIGS["mini21"]       # 2 streams x 2 steps: two batches per prompt branch
    worst, _ = _stream_case(wl, "fp32", mode, 1.3, 0.8, 4, graph=(mode % 2 == 0))
    assert worst <= TOL_FP32


@pytest.mark.parametrize("mode", [0, 2])
def test_stream_modes_bf16(mode):
    wl = MINI_CONFIGS["mini15"]       # 1 stream x 4 steps
    worst_max, worst = _stream_case(wl, "bf16", mode, 1.2, 1.0, 6)
    print(f"mode {mode}: rel_l2 {worst:.3e}, max|g-o|/max|o| {worst_max:.3e}")
    assert worst <= TOL_BF16
    assert worst_max <= TOL_BF16_MAX


def test_option_changes_the_result_and_single_step_ignores_it():
    wl = MINI_CONFIGS["mini15"]
    u = wl["unet"]
    h, w = wl["latent"]
    ctx = cuda(normal(wl["seeds"]["context"], "context", (u["context_len"], u["context_dim"])))
    outs = {}
    for n in (1, 3):
        x = cuda(normal(wl["seeds"]["inputs"], "unet_x", (n, u["in_channels"], h, w)))
        for xf in (0, 1):
            eng = gpu_engine(wl, "bf16", timesteps=list(range(n, 0, -1)), n_streams=1, cross_frame=xf)
            out = torch.empty_like(x)
            eng.unet_forward(x, [700 - 200 * r for r in range(n)], ctx, out)
            torch.cuda.synchronize()
            outs[(n, xf)] = out.cpu().numpy()
            eng.close()
    assert np.array_equal(outs[(1, 0)], outs[(1, 1)])
    assert not np.array_equal(outs[(3, 0)], outs[(3, 1)])
