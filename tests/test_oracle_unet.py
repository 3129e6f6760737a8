"""Pins of oracle/unet.py: every op against brute-force loops written straight from its definition,
degenerate cases with known answers, and the net's wiring against public parameter counts."""
import math

import numpy as np
import pytest
import torch

from oracle import unet as U
from workloads import CONFIGS, make_weights

DT = torch.float64


def _rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=DT)


def _conv_loops(x, w, b, stride):
    c, h, wd = x.shape
    o, _, k, _ = w.shape
    p = k // 2
    ho, wo = (h + 2 * p - k) // stride + 1, (wd + 2 * p - k) // stride + 1
    y = np.zeros((o, ho, wo))
    for oc in range(o):
        for yy in range(ho):
            for xx in range(wo):
                acc = float(b[oc])
                for ci in range(c):
                    for i in range(k):
                        for j in range(k):
                            sy, sx = yy * stride + i - p, xx * stride + j - p
                            if 0 <= sy < h and 0 <= sx < wd:
                                acc += float(w[oc, ci, i, j]) * float(x[ci, sy, sx])
                y[oc, yy, xx] = acc
    return y


@pytest.mark.parametrize("k,stride,h,w", [(3, 1, 5, 4), (3, 2, 6, 4), (3, 2, 5, 7), (1, 1, 3, 5)])
def test_conv_matches_loops(k, stride, h, w):
    x, wt, b = _rand(3, h, w, seed=1), _rand(2, 3, k, k, seed=2), _rand(2, seed=3)
    got = U.conv2d(x, wt, b, stride).numpy()
    np.testing.assert_allclose(got, _conv_loops(x, wt, b, stride), rtol=0, atol=1e-12)


def test_conv_centre_tap_is_a_linear_map():
    x, m, b = _rand(4, 6, 5, seed=4), _rand(3, 4, seed=5), _rand(3, seed=6)
    w = torch.zeros(3, 4, 3, 3, dtype=DT)
    w[:, :, 1, 1] = m
    want = torch.einsum("oc,chw->ohw", m, x) + b[:, None, None]
    np.testing.assert_allclose(U.conv2d(x, w, b).numpy(), want.numpy(), atol=1e-12)


def test_conv_shift_kernel_moves_the_image():
    # a single 1 at tap (0,1) of a 3x3 kernel reads the pixel one row up: out[y,x] = in[y-1,x], zero at the border
    x = _rand(1, 4, 4, seed=7)
    w = torch.zeros(1, 1, 3, 3, dtype=DT)
    w[0, 0, 0, 1] = 1.0
    y = U.conv2d(x, w, torch.zeros(1, dtype=DT))
    assert torch.equal(y[0, 1:], x[0, :-1]) and torch.all(y[0, 0] == 0)


def test_group_norm_matches_loops():
    c, h, w, g = 6, 3, 4, 3
    x, ga, be = _rand(c, h, w, seed=8) * 3 + 1, _rand(c, seed=9), _rand(c, seed=10)
    got = U.group_norm(x, g, ga, be, 1e-5).numpy()
    cg = c // g
    for gi in range(g):
        vals = [float(x[ci, y, xx]) for ci in range(gi * cg, (gi + 1) * cg) for y in range(h) for xx in range(w)]
        mu = sum(vals) / len(vals)
        var = sum((v - mu) ** 2 for v in vals) / len(vals)
        for ci in range(gi * cg, (gi + 1) * cg):
            for y in range(h):
                for xx in range(w):
                    want = (float(x[ci, y, xx]) - mu) / math.sqrt(var + 1e-5) * float(ga[ci]) + float(be[ci])
                    assert abs(got[ci, y, xx] - want) < 1e-12


def test_group_norm_degenerate_single_value_groups():
    x, ga, be = _rand(4, 1, 1, seed=11), _rand(4, seed=12), _rand(4, seed=13)
    np.testing.assert_allclose(U.group_norm(x, 4, ga, be, 1e-5)[:, 0, 0].numpy(), be.numpy(), atol=1e-15)


def test_group_norm_output_statistics():
    x = _rand(8, 5, 5, seed=14) * 7 - 3
    y = U.group_norm(x, 2, torch.ones(8, dtype=DT), torch.zeros(8, dtype=DT), 0.0).reshape(2, -1)
    np.testing.assert_allclose(y.mean(1).numpy(), 0, atol=1e-12)
    np.testing.assert_allclose((y ** 2).mean(1).numpy(), 1, atol=1e-12)


def test_layer_norm_matches_loops():
    x, g, b = _rand(3, 5, seed=15) * 2 + 0.5, _rand(5, seed=16), _rand(5, seed=17)
    got = U.layer_norm(x, g, b).numpy()
    for r in range(3):
        row = [float(v) for v in x[r]]
        mu = sum(row) / 5
        var = sum((v - mu) ** 2 for v in row) / 5
        for j in range(5):
            assert abs(got[r, j] - ((row[j] - mu) / math.sqrt(var + 1e-5) * float(g[j]) + float(b[j]))) < 1e-12


def test_attention_matches_loops():
    tq, tk, heads, d = 5, 7, 2, 3
    q, k, v = _rand(tq, heads * d, seed=18), _rand(tk, heads * d, seed=19), _rand(tk, heads * d, seed=20)
    got = U.attention(q, k, v, heads).numpy()
    for h in range(heads):
        for i in range(tq):
            sc = [sum(float(q[i, h * d + e]) * float(k[j, h * d + e]) for e in range(d)) / math.sqrt(d) for j in range(tk)]
            m = max(sc)
            p = [math.exp(s - m) for s in sc]
            z = sum(p)
            for e in range(d):
                want = sum(p[j] / z * float(v[j, h * d + e]) for j in range(tk))
                assert abs(got[i, h * d + e] - want) < 1e-12


def test_attention_equal_scores_is_mean_of_values():
    k, v = _rand(6, 8, seed=21), _rand(6, 8, seed=22)
    got = U.attention(torch.zeros(4, 8, dtype=DT), k, v, 2)
    np.testing.assert_allclose(got.numpy(), v.mean(0, keepdim=True).expand(4, 8).numpy(), atol=1e-14)


def test_attention_one_hot_selects_a_value_row():
    k = torch.eye(4, dtype=DT) * 200.0
    v = _rand(4, 4, seed=23)
    q = torch.eye(4, dtype=DT)[[2, 0]] * 200.0
    np.testing.assert_allclose(U.attention(q, k, v, 1).numpy(), v[[2, 0]].numpy(), atol=1e-12)


def test_activations_known_values():
    x = torch.tensor([0.0, 1.0, -1.0], dtype=DT)
    # GELU(x) = x Phi(x); Phi(1) = 0.8413447460685429 (standard normal table)
    np.testing.assert_allclose(U.gelu_erf(x).numpy(), [0.0, 0.8413447460685429, -0.15865525393145707], atol=1e-15)
    # SiLU(x) = x sigmoid(x); sigmoid(1) = 0.7310585786300049
    np.testing.assert_allclose(U.silu(x).numpy(), [0.0, 0.7310585786300049, -0.2689414213699951], atol=1e-15)


def test_time_embedding_values():
    e = U.time_embedding(0, 8)
    assert torch.equal(e, torch.tensor([1, 1, 1, 1, 0, 0, 0, 0], dtype=DT))
    e = U.time_embedding(999, 320)
    assert abs(e[0].item() - math.cos(999.0)) < 1e-12 and abs(e[160].item() - math.sin(999.0)) < 1e-12
    f_last = 10000.0 ** (-159.0 / 160.0)
    assert abs(e[159].item() - math.cos(999.0 * f_last)) < 1e-12
    assert abs(e[319].item() - math.sin(999.0 * f_last)) < 1e-12


def test_upsample_nearest():
    x = torch.arange(6, dtype=DT).reshape(1, 2, 3)
    y = U.upsample_nearest2(x)
    assert y.shape == (1, 4, 6)
    for yy in range(4):
        for xx in range(6):
            assert y[0, yy, xx] == x[0, yy // 2, xx // 2]


def test_parameter_counts_match_the_public_nets():
    # 859,520,964 (SD-1.5 U-Net) and 865,910,724 (SD-2.1 U-Net) are the publicly documented sizes of the nets
    # these two workload shapes copy; a missing or mis-sized module in the wiring changes the count.
    assert U.param_count(U.UNetShape.from_dict(CONFIGS[3]["unet"])) == 859_520_964
    assert U.param_count(U.UNetShape.from_dict(CONFIGS[2]["unet"])) == 865_910_724


def _tiny():
    shape = U.UNetShape.from_dict(CONFIGS[1]["unet"])
    blob = make_weights(U.manifest(shape), 77, "fanin", False)
    return shape, blob


def test_every_parameter_reaches_the_output():
    shape, blob = _tiny()
    x, ctx = _rand(4, 8, 8, seed=30), _rand(8, 64, seed=31)
    base = U.unet_single(shape, U.unpack(shape, blob), x, 500, ctx)
    assert base.shape == (4, 8, 8) and torch.isfinite(base).all()
    off = 0
    for name, sh, kind in U.manifest(shape):
        n = math.prod(sh)
        b2 = blob.copy()
        b2[off:off + n] += 0.37
        off += n
        out = U.unet_single(shape, U.unpack(shape, b2), x, 500, ctx)
        assert (out - base).abs().max() > 1e-9, f"{name} does not influence the output"


def test_timestep_and_context_reach_the_output():
    shape, blob = _tiny()
    P = U.unpack(shape, blob)
    x, ctx = _rand(4, 8, 8, seed=32), _rand(8, 64, seed=33)
    base = U.unet_single(shape, P, x, 500, ctx)
    assert (U.unet_single(shape, P, x, 501, ctx) - base).abs().max() > 1e-9
    assert (U.unet_single(shape, P, x, 500, ctx * 1.5) - base).abs().max() > 1e-9


def test_res_block_with_dead_branch_is_the_skip_path():
    P = {"r.norm1.g": torch.ones(4, dtype=DT), "r.norm1.b": torch.zeros(4, dtype=DT),
         "r.conv1.w": _rand(6, 4, 3, 3, seed=34), "r.conv1.b": _rand(6, seed=35),
         "r.temb.w": _rand(6, 8, seed=36), "r.temb.b": _rand(6, seed=37),
         "r.norm2.g": torch.ones(6, dtype=DT), "r.norm2.b": torch.zeros(6, dtype=DT),
         "r.conv2.w": torch.zeros(6, 6, 3, 3, dtype=DT), "r.conv2.b": torch.zeros(6, dtype=DT),
         "r.skip.w": _rand(6, 4, 1, 1, seed=38), "r.skip.b": _rand(6, seed=39)}
    x = _rand(4, 5, 5, seed=40)
    want = torch.einsum("oc,chw->ohw", P["r.skip.w"][:, :, 0, 0], x) + P["r.skip.b"][:, None, None]
    np.testing.assert_allclose(U.res_block(P, "r", x, _rand(8, seed=41), 2).numpy(), want.numpy(), atol=1e-12)


def test_batch_rows_are_independent():
    shape, blob = _tiny()
    net = U.UNet(shape, blob)
    x, ctx = _rand(3, 4, 8, 8, seed=42), _rand(8, 64, seed=43)
    full = net(x, [999, 499, 10], ctx)
    alone = net(x[1:2], [499], ctx)
    assert torch.equal(full[1], alone[0])
    assert net.evaluations == 4
