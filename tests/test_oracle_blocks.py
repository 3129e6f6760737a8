"""Definition-level pins of the blocks of oracle/unet.py.

The paper treats the U-Net as a black box (Sec. 3.1), so the written definition of the net is the specification.
Here that definition is written out a second time as scalar Python loops over nested lists - no tensor library, no
function of oracle/ - for one ResBlock (time embedding, 1x1 skip), one transformer block and the whole net at a
very small shape, and the oracle must agree to 1e-12.  The second half plants, in the oracle and on the CPU, each
of the wiring mistakes such a definition invites and checks that the pins notice every one of them.
"""
import math
from unittest import mock

import numpy as np
import pytest
import torch

from oracle import unet as U

DT = torch.float64


def _rand(*shape, seed=0, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=DT) * scale


# ------------------------------------------------------------------------------------------------
# the definition in loops.  Feature maps are lists [c][y][x]; token matrices are lists [t][c].
# ------------------------------------------------------------------------------------------------
def L(t):
    return t.tolist()


def l_silu(v):
    return v / (1.0 + math.exp(-v))


def l_gelu(v):
    return 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))


def l_conv(x, w, b, stride=1):
    """Zero-padded k x k correlation, pad k//2: y[o][y][x] = b[o] + sum w[o][c][i][j] x[c][y*stride+i-p][x*stride+j-p]."""
    c, h, wd = len(x), len(x[0]), len(x[0][0])
    k = len(w[0][0])
    p = k // 2
    ho, wo = (h + 2 * p - k) // stride + 1, (wd + 2 * p - k) // stride + 1
    y = [[[0.0] * wo for _ in range(ho)] for _ in range(len(w))]
    for o in range(len(w)):
        for yy in range(ho):
            for xx in range(wo):
                acc = b[o] if b is not None else 0.0
                for ci in range(c):
                    for i in range(k):
                        sy = yy * stride + i - p
                        if not 0 <= sy < h:
                            continue
                        for j in range(k):
                            sx = xx * stride + j - p
                            if 0 <= sx < wd:
                                acc += w[o][ci][i][j] * x[ci][sy][sx]
                y[o][yy][xx] = acc
    return y


def l_group_norm(x, groups, g, b, eps):
    c, h, wd = len(x), len(x[0]), len(x[0][0])
    cg = c // groups
    y = [[[0.0] * wd for _ in range(h)] for _ in range(c)]
    for gi in range(groups):
        vals = [x[ci][yy][xx] for ci in range(gi * cg, (gi + 1) * cg) for yy in range(h) for xx in range(wd)]
        mu = sum(vals) / len(vals)
        var = sum((v - mu) ** 2 for v in vals) / len(vals)
        for ci in range(gi * cg, (gi + 1) * cg):
            for yy in range(h):
                for xx in range(wd):
                    y[ci][yy][xx] = (x[ci][yy][xx] - mu) / math.sqrt(var + eps) * g[ci] + b[ci]
    return y


def l_layer_norm(rows, g, b, eps=1e-5):
    out = []
    for r in rows:
        mu = sum(r) / len(r)
        var = sum((v - mu) ** 2 for v in r) / len(r)
        out.append([(v - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, v in enumerate(r)])
    return out


def l_linear(rows, w, b=None):
    return [[sum(w[o][i] * r[i] for i in range(len(r))) + (b[o] if b is not None else 0.0) for o in range(len(w))]
            for r in rows]


def l_attention(q, k, v, heads):
    c = len(q[0])
    d = c // heads
    out = [[0.0] * c for _ in q]
    for h in range(heads):
        for i, qi in enumerate(q):
            s = [sum(qi[h * d + e] * kj[h * d + e] for e in range(d)) / math.sqrt(d) for kj in k]
            m = max(s)
            p = [math.exp(v_ - m) for v_ in s]
            z = sum(p)
            for e in range(d):
                out[i][h * d + e] = sum(p[j] / z * v[j][h * d + e] for j in range(len(k)))
    return out


def l_map_silu(x):
    return [[[l_silu(v) for v in row] for row in ch] for ch in x]


def l_add(a, b):
    return [[[a[c][y][x] + b[c][y][x] for x in range(len(a[0][0]))] for y in range(len(a[0]))] for c in range(len(a))]


def l_res_block(P, p, x, temb, groups):
    """GN(1e-5), SiLU, conv3x3; + Linear(SiLU(temb)) per channel; GN(1e-5), SiLU, conv3x3; + x (through a 1x1
    convolution when the block changes the width)."""
    h = l_conv(l_map_silu(l_group_norm(x, groups, P[p + ".norm1.g"], P[p + ".norm1.b"], 1e-5)),
               P[p + ".conv1.w"], P[p + ".conv1.b"])
    tb = l_linear([[l_silu(v) for v in temb]], P[p + ".temb.w"], P[p + ".temb.b"])[0]
    h = [[[v + tb[c] for v in row] for row in ch] for c, ch in enumerate(h)]
    h = l_conv(l_map_silu(l_group_norm(h, groups, P[p + ".norm2.g"], P[p + ".norm2.b"], 1e-5)),
               P[p + ".conv2.w"], P[p + ".conv2.b"])
    skip = l_conv(x, P[p + ".skip.w"], P[p + ".skip.b"]) if (p + ".skip.w") in P else x
    return l_add(skip, h)


def l_transformer(P, p, x, ctx, heads, groups):
    """GN(1e-6), proj_in on tokens; h += attn1(LN h); h += attn2(LN h, ctx); h += FF(LN h); proj_out; + x.
    q/k/v have no bias, the output projections have one; FF = Linear(C, 8C) -> first half * GELU(second half)
    -> Linear(4C, C)."""
    c, hh, ww = len(x), len(x[0]), len(x[0][0])
    gn = l_group_norm(x, groups, P[p + ".norm.g"], P[p + ".norm.b"], 1e-6)
    tok = [[gn[ci][yy][xx] for ci in range(c)] for yy in range(hh) for xx in range(ww)]
    h = l_linear(tok, P[p + ".proj_in.w"], P[p + ".proj_in.b"])
    n = l_layer_norm(h, P[p + ".ln1.g"], P[p + ".ln1.b"])
    a = l_attention(l_linear(n, P[p + ".attn1.q.w"]), l_linear(n, P[p + ".attn1.k.w"]),
                    l_linear(n, P[p + ".attn1.v.w"]), heads)
    a = l_linear(a, P[p + ".attn1.o.w"], P[p + ".attn1.o.b"])
    h = [[u + v for u, v in zip(r, s)] for r, s in zip(h, a)]
    n = l_layer_norm(h, P[p + ".ln2.g"], P[p + ".ln2.b"])
    a = l_attention(l_linear(n, P[p + ".attn2.q.w"]), l_linear(ctx, P[p + ".attn2.k.w"]),
                    l_linear(ctx, P[p + ".attn2.v.w"]), heads)
    a = l_linear(a, P[p + ".attn2.o.w"], P[p + ".attn2.o.b"])
    h = [[u + v for u, v in zip(r, s)] for r, s in zip(h, a)]
    n = l_layer_norm(h, P[p + ".ln3.g"], P[p + ".ln3.b"])
    u = l_linear(n, P[p + ".ff.in.w"], P[p + ".ff.in.b"])
    inner = len(u[0]) // 2
    u = [[r[i] * l_gelu(r[inner + i]) for i in range(inner)] for r in u]
    f = l_linear(u, P[p + ".ff.out.w"], P[p + ".ff.out.b"])
    h = [[a_ + b_ for a_, b_ in zip(r, s)] for r, s in zip(h, f)]
    h = l_linear(h, P[p + ".proj_out.w"], P[p + ".proj_out.b"])
    return [[[x[ci][yy][xx] + h[yy * ww + xx][ci] for xx in range(ww)] for yy in range(hh)] for ci in range(c)]


def l_unet(shape, P, x, t, ctx):
    ch = shape.block_channels
    nl, g = len(ch), shape.norm_groups
    half = ch[0] // 2
    emb = [math.cos(t * math.exp(-math.log(10000.0) * j / half)) for j in range(half)] + \
          [math.sin(t * math.exp(-math.log(10000.0) * j / half)) for j in range(half)]
    e1 = l_linear([emb], P["time.lin1.w"], P["time.lin1.b"])[0]
    temb = l_linear([[l_silu(v) for v in e1]], P["time.lin2.w"], P["time.lin2.b"])[0]
    h = l_conv(x, P["conv_in.w"], P["conv_in.b"])
    skips = [h]
    for l in range(nl):
        for j in range(shape.layers_per_block):
            h = l_res_block(P, f"down.{l}.res.{j}", h, temb, g)
            if shape.attn_levels[l]:
                h = l_transformer(P, f"down.{l}.attn.{j}", h, ctx, shape.heads(ch[l]), g)
            skips.append(h)
        if l != nl - 1:
            h = l_conv(h, P[f"down.{l}.downsample.w"], P[f"down.{l}.downsample.b"], 2)
            skips.append(h)
    h = l_res_block(P, "mid.res.0", h, temb, g)
    if shape.mid_attention:
        h = l_transformer(P, "mid.attn", h, ctx, shape.heads(ch[-1]), g)
    h = l_res_block(P, "mid.res.1", h, temb, g)
    for l in reversed(range(nl)):
        for j in range(shape.layers_per_block + 1):
            h = l_res_block(P, f"up.{l}.res.{j}", h + skips.pop(), temb, g)   # list concat = channel concat, h first
            if shape.attn_levels[l]:
                h = l_transformer(P, f"up.{l}.attn.{j}", h, ctx, shape.heads(ch[l]), g)
        if l != 0:
            up = [[[chn[yy // 2][xx // 2] for xx in range(2 * len(chn[0]))] for yy in range(2 * len(chn))] for chn in h]
            h = l_conv(up, P[f"up.{l}.upsample.w"], P[f"up.{l}.upsample.b"])
    assert not skips
    h = l_map_silu(l_group_norm(h, g, P["out.norm.g"], P["out.norm.b"], 1e-5))
    return l_conv(h, P["conv_out.w"], P["conv_out.b"])


# ------------------------------------------------------------------------------------------------
# cases.  Inputs are small in magnitude so that the norm epsilons (1e-5 / 1e-6) carry weight, and the norm
# scales and shifts are random (the workloads use 1 and 0, which would hide a dropped or misplaced affine term).
# ------------------------------------------------------------------------------------------------
def _params(entries, seed):
    P = {}
    for i, (name, shape, kind) in enumerate(entries):
        t = _rand(*shape, seed=seed + i, scale=0.3 if kind == "weight" else 0.5)
        P[name] = t + 1.0 if kind == "gamma" else t
    return P


def _lists(P):
    return {k: L(v) for k, v in P.items()}


RES_CASES = {"skip1x1": dict(cin=6, cout=4, temb=8, groups=2, h=5, w=4),
             "identity": dict(cin=4, cout=4, temb=8, groups=2, h=4, w=3)}
TF_CASE = dict(c=8, heads=2, groups=4, h=3, w=4, lctx=3, dctx=5)
MICRO = U.UNetShape(in_channels=2, block_channels=(8, 16), layers_per_block=1, attn_levels=(0, 1), num_heads=0,
                    head_dim=8, mid_attention=1, context_len=3, context_dim=5, norm_groups=4)


def _res_inputs(case):
    k = RES_CASES[case]
    P = _params(U._res_entries("r", k["cin"], k["cout"], k["temb"]), 100)
    x = _rand(k["cin"], k["h"], k["w"], seed=1, scale=3e-3) + 0.01
    temb = _rand(k["temb"], seed=2)
    return P, x, temb


def _tf_inputs():
    k = TF_CASE
    P = _params(U._tf_entries("t", k["c"], k["dctx"]), 200)
    x = _rand(k["c"], k["h"], k["w"], seed=3, scale=1e-3) + 0.02
    ctx = _rand(k["lctx"], k["dctx"], seed=4)
    return P, x, ctx


def _micro_inputs():
    P = _params(U.manifest(MICRO), 300)
    x = _rand(2, 4, 4, seed=5)
    ctx = _rand(MICRO.context_len, MICRO.context_dim, seed=6)
    return P, x, ctx


def _res_gap(case):
    P, x, temb = _res_inputs(case)
    groups = RES_CASES[case]["groups"]
    got = U.res_block(P, "r", x, temb, groups).numpy()
    want = np.array(l_res_block(_lists(P), "r", L(x), L(temb), groups))
    return float(np.abs(got - want).max() / np.abs(want).max())


def _tf_gap():
    P, x, ctx = _tf_inputs()
    got = U.transformer(P, "t", x, ctx, TF_CASE["heads"], TF_CASE["groups"]).numpy()
    want = np.array(l_transformer(_lists(P), "t", L(x), L(ctx), TF_CASE["heads"], TF_CASE["groups"]))
    return float(np.abs(got - want).max() / np.abs(want).max())


_MICRO_WANT = {}


def _micro_gap():
    P, x, ctx = _micro_inputs()
    if "v" not in _MICRO_WANT:
        _MICRO_WANT["v"] = np.array(l_unet(MICRO, _lists(P), L(x), 437, L(ctx)))
    got = U.unet_single(MICRO, P, x, 437, ctx).numpy()
    return float(np.abs(got - _MICRO_WANT["v"]).max() / np.abs(_MICRO_WANT["v"]).max())


@pytest.mark.parametrize("case", sorted(RES_CASES))
def test_res_block_with_time_embedding_matches_loops(case):
    assert _res_gap(case) < 1e-12


def test_transformer_block_matches_loops():
    assert _tf_gap() < 1e-12


def test_whole_net_at_micro_shape_matches_loops():
    # two levels, a stride-2 convolution, transformer blocks at the deep level and in the middle, an upsampling
    # convolution, and two skips of equal width and size popped one after the other at level 0
    assert U.param_count(MICRO) == sum(math.prod(s) for _, s, _ in U.manifest(MICRO))
    assert _micro_gap() < 1e-12


# ------------------------------------------------------------------------------------------------
# planted mistakes (in the oracle, on the CPU): each must move at least one pin far beyond its tolerance
# ------------------------------------------------------------------------------------------------
_ORIG = {"res_block": U.res_block, "silu": U.silu, "group_norm": U.group_norm}


def _silu_skipping_vectors(v):
    return v if v.dim() == 1 else _ORIG["silu"](v)      # the only vector SiLU ever sees is the time embedding


def _res_block_temb_before_conv1(P, p, x, temb, groups):
    if x.shape[0] != P[p + ".temb.w"].shape[0]:
        return _ORIG["res_block"](P, p, x, temb, groups)
    h = U.silu(U.group_norm(x, groups, P[p + ".norm1.g"], P[p + ".norm1.b"], 1e-5))
    h = h + U._linear(U.silu(temb), P[p + ".temb.w"], P[p + ".temb.b"])[:, None, None]
    h = U.conv2d(h, P[p + ".conv1.w"], P[p + ".conv1.b"])
    h = U.conv2d(U.silu(U.group_norm(h, groups, P[p + ".norm2.g"], P[p + ".norm2.b"], 1e-5)),
                 P[p + ".conv2.w"], P[p + ".conv2.b"])
    return x + h


def _group_norm_eps_swapped(x, groups, g, b, eps):
    return _ORIG["group_norm"](x, groups, g, b, {1e-5: 1e-6, 1e-6: 1e-5}[eps])


def _gelu_on_the_other_half(P):
    Q = dict(P)
    for k in P:
        if k.endswith(".ff.in.w") or k.endswith(".ff.in.b"):
            half = P[k].shape[0] // 2
            Q[k] = torch.cat([P[k][half:], P[k][:half]], dim=0)
    return Q


def _micro_net_by_hand(P, x, ctx, swap_level0_skips):
    """The micro net wired by hand from the oracle's blocks; optionally with the two level-0 skips, which have the
    same width and size, handed out in push order instead of pop order."""
    s, g = MICRO, MICRO.norm_groups
    heads = s.heads(s.block_channels[1])
    e = U.time_embedding(437, s.block_channels[0])
    temb = U._linear(U.silu(U._linear(e, P["time.lin1.w"], P["time.lin1.b"])), P["time.lin2.w"], P["time.lin2.b"])
    h0 = U.conv2d(x, P["conv_in.w"], P["conv_in.b"])
    h1 = U.res_block(P, "down.0.res.0", h0, temb, g)
    h2 = U.conv2d(h1, P["down.0.downsample.w"], P["down.0.downsample.b"], stride=2)
    h3 = U.transformer(P, "down.1.attn.0", U.res_block(P, "down.1.res.0", h2, temb, g), ctx, heads, g)
    m = U.res_block(P, "mid.res.0", h3, temb, g)
    m = U.transformer(P, "mid.attn", m, ctx, heads, g)
    m = U.res_block(P, "mid.res.1", m, temb, g)
    u = U.transformer(P, "up.1.attn.0", U.res_block(P, "up.1.res.0", torch.cat([m, h3]), temb, g), ctx, heads, g)
    u = U.transformer(P, "up.1.attn.1", U.res_block(P, "up.1.res.1", torch.cat([u, h2]), temb, g), ctx, heads, g)
    u = U.conv2d(U.upsample_nearest2(u), P["up.1.upsample.w"], P["up.1.upsample.b"])
    first, second = (h0, h1) if swap_level0_skips else (h1, h0)
    u = U.res_block(P, "up.0.res.0", torch.cat([u, first]), temb, g)
    u = U.res_block(P, "up.0.res.1", torch.cat([u, second]), temb, g)
    u = U.silu(U.group_norm(u, g, P["out.norm.g"], P["out.norm.b"], 1e-5))
    return U.conv2d(u, P["conv_out.w"], P["conv_out.b"]).numpy()


def test_the_pins_notice_silu_missing_on_the_time_embedding():
    _micro_gap()   # the loop result is cached from the unpatched run
    with mock.patch.object(U, "silu", _silu_skipping_vectors):
        assert _res_gap("skip1x1") > 1e-3 and _micro_gap() > 1e-3


def test_the_pins_notice_the_time_embedding_added_before_conv1():
    _micro_gap()
    with mock.patch.object(U, "res_block", _res_block_temb_before_conv1):
        assert _res_gap("identity") > 1e-3 and _micro_gap() > 1e-3


def test_the_pins_notice_swapped_group_norm_epsilons():
    with mock.patch.object(U, "group_norm", _group_norm_eps_swapped):
        assert _res_gap("skip1x1") > 1e-3
        assert _tf_gap() > 1e-3


def test_the_pins_notice_swapped_geglu_halves():
    P, x, ctx = _tf_inputs()
    got = U.transformer(_gelu_on_the_other_half(P), "t", x, ctx, TF_CASE["heads"], TF_CASE["groups"]).numpy()
    want = np.array(l_transformer(_lists(P), "t", L(x), L(ctx), TF_CASE["heads"], TF_CASE["groups"]))
    assert np.abs(got - want).max() / np.abs(want).max() > 1e-3


def test_the_pins_notice_equal_width_skips_popped_in_the_wrong_order():
    assert _micro_gap() < 1e-12
    P, x, ctx = _micro_inputs()
    want = _MICRO_WANT["v"]
    right = _micro_net_by_hand(P, x, ctx, False)
    wrong = _micro_net_by_hand(P, x, ctx, True)
    assert np.abs(right - want).max() / np.abs(want).max() < 1e-12
    assert np.abs(wrong - want).max() / np.abs(want).max() > 1e-3
