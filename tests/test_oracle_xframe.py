"""Pins of the oracle's Stream Batch cross-frame attention (Sec. 3.2 of the paper: K_Batch / V_Batch and the Attn
equation built on them): special cases that reduce to the plain path, set-invariance, and a brute-force loop over the
keys of all rows written straight from the softmax definition."""
import math

import numpy as np
import pytest
import torch

from oracle import stream as S
from oracle import unet as U
from workloads import CONFIGS, make_weights

DT = torch.float64


def _rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=DT)


def _tiny():
    shape = U.UNetShape.from_dict(CONFIGS[1]["unet"])
    blob = make_weights(U.manifest(shape), 77, "fanin", False)
    return shape, blob


def _tf_params(c, dctx, seed):
    names = {".norm.g": (c,), ".norm.b": (c,), ".proj_in.w": (c, c), ".proj_in.b": (c,),
             ".ln1.g": (c,), ".ln1.b": (c,), ".attn1.q.w": (c, c), ".attn1.k.w": (c, c), ".attn1.v.w": (c, c),
             ".attn1.o.w": (c, c), ".attn1.o.b": (c,), ".ln2.g": (c,), ".ln2.b": (c,),
             ".attn2.q.w": (c, c), ".attn2.k.w": (c, dctx), ".attn2.v.w": (c, dctx), ".attn2.o.w": (c, c),
             ".attn2.o.b": (c,), ".ln3.g": (c,), ".ln3.b": (c,), ".ff.in.w": (8 * c, c), ".ff.in.b": (8 * c,),
             ".ff.out.w": (c, 4 * c), ".ff.out.b": (c,), ".proj_out.w": (c, c), ".proj_out.b": (c,)}
    return {"t" + k: _rand(*sh, seed=seed + i) * 0.5 for i, (k, sh) in enumerate(names.items())}


def test_single_row_reduces_to_the_plain_path():
    shape, blob = _tiny()
    x, ctx = _rand(1, 4, 8, 8, seed=1), _rand(8, 64, seed=2)
    assert torch.equal(U.UNet(shape, blob, cross_frame=True)(x, [417], ctx), U.UNet(shape, blob)(x, [417], ctx))


def test_identical_rows_change_nothing():
    # n copies of the same keys and values leave every softmax-weighted mean where it was
    shape, blob = _tiny()
    x1, ctx = _rand(4, 8, 8, seed=3), _rand(8, 64, seed=4)
    plain = U.UNet(shape, blob)(x1[None], [500], ctx)[0]
    got = U.UNet(shape, blob, cross_frame=True)(torch.stack([x1, x1, x1]), [500, 500, 500], ctx)
    for r in range(3):
        np.testing.assert_allclose(got[r].numpy(), plain.numpy(), rtol=0, atol=1e-11)


def test_rows_form_a_set():
    # the keys of a batch are a set: a different row order permutes the outputs and changes none of them
    shape, blob = _tiny()
    x, ctx, t = _rand(3, 4, 8, 8, seed=5), _rand(8, 64, seed=6), [999, 499, 10]
    net = U.UNet(shape, blob, cross_frame=True)
    base = net(x, t, ctx)
    perm = [2, 0, 1]
    got = net(x[perm], [t[i] for i in perm], ctx)
    for new, old in enumerate(perm):
        np.testing.assert_allclose(got[new].numpy(), base[old].numpy(), rtol=0, atol=1e-11)


def test_rows_are_coupled_only_when_asked():
    shape, blob = _tiny()
    x, ctx, t = _rand(2, 4, 8, 8, seed=7), _rand(8, 64, seed=8), [800, 300]
    x2 = x.clone()
    x2[1] += 0.5
    on, off = U.UNet(shape, blob, cross_frame=True), U.UNet(shape, blob)
    assert (on(x, t, ctx)[0] - on(x2, t, ctx)[0]).abs().max() > 1e-9      # row 1 reaches row 0
    assert torch.equal(off(x, t, ctx)[0], off(x2, t, ctx)[0])             # and does not without it
    assert (on(x, t, ctx)[0] - off(x, t, ctx)[0]).abs().max() > 1e-9


def test_self_attention_over_the_batch_matches_loops():
    # One transformer block on three rows.  Expected: the block evaluated row by row with the plain path, except that
    # the self-attention term is replaced by an explicit loop over the keys of ALL rows (softmax written out).
    c, heads, hw, n, groups = 8, 2, (2, 3), 3, 2
    d = c // heads
    P = _tf_params(c, 6, seed=100)
    xs = [_rand(c, *hw, seed=200 + r) for r in range(n)]
    ctx = _rand(5, 6, seed=300)
    got = U.transformer_rows(P, "t", xs, ctx, heads, groups, True)

    toks, qs, ks, vs = [], [], [], []
    for x in xs:
        h = U.group_norm(x, groups, P["t.norm.g"], P["t.norm.b"], 1e-6).reshape(c, -1).T
        h = h @ P["t.proj_in.w"].T + P["t.proj_in.b"]
        nrm = U.layer_norm(h, P["t.ln1.g"], P["t.ln1.b"])
        toks.append(h)
        qs.append((nrm @ P["t.attn1.q.w"].T).numpy())
        ks.append((nrm @ P["t.attn1.k.w"].T).numpy())
        vs.append((nrm @ P["t.attn1.v.w"].T).numpy())
    T = hw[0] * hw[1]
    for r in range(n):
        att = np.zeros((T, c))
        for tq in range(T):
            for hd in range(heads):
                cols = range(hd * d, (hd + 1) * d)
                scores = []
                for rr in range(n):                       # keys of every row of the batch, in batch order
                    for tk in range(T):
                        scores.append(sum(qs[r][tq, j] * ks[rr][tk, j] for j in cols) / math.sqrt(d))
                m = max(scores)
                w = [math.exp(v - m) for v in scores]
                z = sum(w)
                for j in cols:
                    att[tq, j] = sum(w[rr * T + tk] * vs[rr][tk, j] for rr in range(n) for tk in range(T)) / z
        # the rest of the block on this row alone, from the plain single-row function with the self-attention
        # output substituted: run it with attn1 made the identity on a precomputed value
        h = toks[r] + torch.as_tensor(att) @ P["t.attn1.o.w"].T + P["t.attn1.o.b"]
        nrm = U.layer_norm(h, P["t.ln2.g"], P["t.ln2.b"])
        a2 = U.attention(nrm @ P["t.attn2.q.w"].T, ctx @ P["t.attn2.k.w"].T, ctx @ P["t.attn2.v.w"].T, heads)
        h = h + a2 @ P["t.attn2.o.w"].T + P["t.attn2.o.b"]
        nrm = U.layer_norm(h, P["t.ln3.g"], P["t.ln3.b"])
        u = nrm @ P["t.ff.in.w"].T + P["t.ff.in.b"]
        u = u[:, :4 * c] * U.gelu_erf(u[:, 4 * c:])
        h = h + u @ P["t.ff.out.w"].T + P["t.ff.out.b"]
        h = h @ P["t.proj_out.w"].T + P["t.proj_out.b"]
        want = xs[r] + h.T.reshape(c, *hw)
        np.testing.assert_allclose(got[r].numpy(), want.numpy(), rtol=0, atol=1e-11)


def test_plain_transformer_is_the_one_row_case():
    c, heads, groups = 8, 2, 2
    P = _tf_params(c, 6, seed=400)
    x, ctx = _rand(c, 3, 3, seed=500), _rand(5, 6, seed=501)
    assert torch.equal(U.transformer(P, "t", x, ctx, heads, groups),
                       U.transformer_rows(P, "t", [x], ctx, heads, groups, True)[0])


@pytest.mark.parametrize("mode", [S.MODE_NONE, S.MODE_CFG, S.MODE_SELF, S.MODE_ONETIME])
def test_single_step_stream_is_unchanged(mode):
    # with n = 1 every batch is one row, so the whole Stream Batch step must not notice the option
    shape, blob = _tiny()
    wl = dict(CONFIGS[1])
    noise = _rand(1, 1, 4, 8, 8, seed=600)
    ctx, neg = _rand(8, 64, seed=601), _rand(8, 64, seed=602)
    outs = []
    for xf in (False, True):
        sb = S.StreamBatch(U.UNet(shape, blob, cross_frame=xf), [500], noise, mode=mode, gamma=1.3, delta=0.8)
        outs.append([sb.step(_rand(1, 4, 8, 8, seed=610 + k), ctx, neg)[0] for k in range(2)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_stream_batch_rows_of_a_call_share_keys_but_streams_do_not():
    # two streams: stream 1's frames must not reach stream 0's outputs (each stream is its own batch)
    shape, blob = _tiny()
    ts = [800, 300]
    noise = _rand(2, 2, 4, 8, 8, seed=700)
    ctx = _rand(8, 64, seed=701)
    frames = [_rand(2, 4, 8, 8, seed=710 + k) for k in range(3)]
    def run(alter):
        sb = S.StreamBatch(U.UNet(shape, blob, cross_frame=True), ts, noise)
        outs = []
        for f in frames:
            f = f.clone()
            if alter:
                f[1] += 0.3
            outs.append(sb.step(f, ctx)[0])
        return outs
    for a, b in zip(run(False), run(True)):
        assert torch.equal(a[0], b[0])
        assert (a[1] - b[1]).abs().max() > 1e-9
