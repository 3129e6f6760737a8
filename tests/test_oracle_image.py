"""Pins of oracle/image.py (the tiny autoencoder around the U-Net): the definition written a second time as scalar
Python loops over nested lists, closed forms and degenerate cases, and planted wiring mistakes that the pins must
notice.  The paper only names the autoencoder, so the written definition is the specification."""
import math
from unittest import mock

import numpy as np
import pytest
import torch

from oracle import image as I
from test_oracle_blocks import L, l_add, l_conv

DT = torch.float64
W = 2   # width of the loop cases (the definition has one width parameter; the workloads use 64)


def _params(width, seed, scale=0.4):
    g = torch.Generator().manual_seed(seed)
    P = {}
    for name, shape, kind in I.manifest(width):
        P[name] = torch.randn(*shape, generator=g, dtype=DT) * (scale if kind == "weight" else 0.2)
    return P


def l_relu(x):
    return [[[v if v > 0.0 else 0.0 for v in row] for row in ch] for ch in x]


def l_block(P, p, x):
    h = l_relu(l_conv(x, P[p + ".a.w"], P[p + ".a.b"]))
    h = l_relu(l_conv(h, P[p + ".b.w"], P[p + ".b.b"]))
    h = l_conv(h, P[p + ".c.w"], P[p + ".c.b"])
    return l_relu(l_add(h, x))


def l_encode(P, img):
    hh, ww = len(img), len(img[0])
    x = [[[img[y][xx][c] / 255.0 for xx in range(ww)] for y in range(hh)] for c in range(3)]
    x = l_conv(x, P["enc.in.w"], P["enc.in.b"])
    x = l_block(P, "enc.0.block.0", x)
    for s in (1, 2, 3):
        x = l_conv(x, P[f"enc.{s}.down.w"], None, 2)
        for j in range(3):
            x = l_block(P, f"enc.{s}.block.{j}", x)
    return l_conv(x, P["enc.out.w"], P["enc.out.b"])


def l_decode(P, z):
    x = [[[3.0 * math.tanh(v / 3.0) for v in row] for row in ch] for ch in z]
    x = l_relu(l_conv(x, P["dec.in.w"], P["dec.in.b"]))
    for s in (0, 1, 2):
        for j in range(3):
            x = l_block(P, f"dec.{s}.block.{j}", x)
        up = [[[ch[y // 2][xx // 2] for xx in range(2 * len(ch[0]))] for y in range(2 * len(ch))] for ch in x]
        x = l_conv(up, P[f"dec.{s}.up.w"], None)
    x = l_block(P, "dec.3.block.0", x)
    x = l_conv(x, P["dec.out.w"], P["dec.out.b"])
    return [[[min(max(v, 0.0), 1.0) for v in row] for row in ch] for ch in x]


def _lists(P):
    return {k: L(v) for k, v in P.items()}


def _image(h, w, seed):
    return np.random.default_rng(seed).integers(0, 256, size=(h, w, 3), dtype=np.uint8)


_CACHE = {}


def _encode_gap():
    P = _params(W, 1)
    img = _image(16, 24, 2)
    if "enc" not in _CACHE:
        _CACHE["enc"] = np.array(l_encode(_lists(P), img.tolist()))
    got = I.encode(P, img).numpy()
    assert got.shape == (4, 2, 3)
    return float(np.abs(got - _CACHE["enc"]).max() / np.abs(_CACHE["enc"]).max())


def _decode_gap():
    P = _params(W, 3, scale=0.25)
    z = torch.randn(4, 2, 1, generator=torch.Generator().manual_seed(4), dtype=DT) * 2.5
    if "dec" not in _CACHE:
        _CACHE["dec"] = np.array(l_decode(_lists(P), L(z)))
    got = I.decode(P, z).numpy()
    assert got.shape == (3, 16, 8)
    want = _CACHE["dec"]
    assert 0.0 < want.min() + 1e-9 and ((want > 0.02) & (want < 0.98)).mean() > 0.2   # not all clamped away
    return float(np.abs(got - want).max())


def test_block_matches_loops():
    P = _params(3, 5)
    x = torch.randn(3, 4, 5, generator=torch.Generator().manual_seed(6), dtype=DT)
    got = I.block(P, "enc.0.block.0", x).numpy()
    want = np.array(l_block(_lists(P), "enc.0.block.0", L(x)))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_encoder_matches_loops():
    assert _encode_gap() < 1e-12


def test_decoder_matches_loops():
    assert _decode_gap() < 1e-12


def test_parameter_count_closed_form():
    for w in (2, 64):
        blk = 3 * (w * w * 9 + w)
        enc = (w * 27 + w) + 10 * blk + 3 * w * w * 9 + (4 * w * 9 + 4)
        dec = (w * 36 + w) + 10 * blk + 3 * w * w * 9 + (3 * w * 9 + 3)
        assert I.param_count(w) == enc + dec
    assert I.param_count(64) == 1_222_532 + 1_222_531


def test_dead_block_is_a_relu():
    P = _params(3, 7)
    P["enc.0.block.0.c.w"].zero_()
    P["enc.0.block.0.c.b"].zero_()
    x = torch.randn(3, 4, 4, generator=torch.Generator().manual_seed(8), dtype=DT)
    assert torch.equal(I.block(P, "enc.0.block.0", x), torch.clamp(x, min=0.0))


def test_decoder_saturates_large_latents_and_passes_small_ones():
    P = _params(W, 9, scale=0.25)
    z = torch.randn(4, 1, 2, generator=torch.Generator().manual_seed(10), dtype=DT)
    big1, big2 = I.decode(P, z * 1e6), I.decode(P, z * 3e6)      # 3 tanh(x/3) = +-3 for both
    assert torch.equal(big1, big2)
    sat = I.decode(P, 1e3 * torch.sign(z))
    assert torch.allclose(big1, sat, atol=1e-12)
    with mock.patch.object(torch, "tanh", lambda v: v):            # without the squashing the two would differ
        assert not torch.equal(I.decode(P, z * 1e6), I.decode(P, z * 3e6))


def test_constant_image_through_bias_only_encoder():
    # all weights zero: every convolution returns its bias, every Block ReLU(bias_c + input)
    P = {k: torch.zeros_like(v) for k, v in _params(W, 11).items()}
    P["enc.out.b"] = torch.tensor([0.5, -1.0, 2.0, 0.0], dtype=DT)
    lat = I.encode(P, _image(8, 16, 12))
    assert lat.shape == (4, 1, 2)
    assert torch.equal(lat, P["enc.out.b"][:, None, None].expand(4, 1, 2))


def test_u8_conversion():
    img = torch.tensor([0.0, 0.5 / 255, 1.5 / 255, 2.5 / 255, 0.999, 1.0], dtype=DT).reshape(1, 1, 6).expand(3, 1, 6)
    assert I.to_u8(img)[0, :, 0].tolist() == [0, 0, 2, 2, 255, 255]      # round half to even


# ---- planted mistakes (in the oracle, on the CPU)
_ORIG_BLOCK = I.block


def _block_relu_before_the_skip(P, p, x):
    h = I.relu(I.conv3x3(x, P[p + ".a.w"], P[p + ".a.b"]))
    h = I.relu(I.conv3x3(h, P[p + ".b.w"], P[p + ".b.b"]))
    return I.relu(I.conv3x3(h, P[p + ".c.w"], P[p + ".c.b"])) + x


def test_the_pins_notice_relu_applied_before_the_skip_sum():
    _encode_gap(), _decode_gap()
    with mock.patch.object(I, "block", _block_relu_before_the_skip):
        assert _encode_gap() > 1e-3 and _decode_gap() > 1e-3


def test_the_pins_notice_a_missing_relu_after_the_decoders_first_convolution():
    _decode_gap()
    calls = {"n": 0}
    real = I.relu

    def relu_skipping_first(x):
        calls["n"] += 1
        return x if calls["n"] == 1 else real(x)
    with mock.patch.object(I, "relu", relu_skipping_first):
        assert _decode_gap() > 1e-3


def test_the_pins_notice_upsampling_after_instead_of_before_the_stage_convolution():
    _decode_gap()
    real_conv, real_up = I.conv3x3, I.upsample_nearest2

    def conv_then_upsample(x, w, b=None, stride=1):
        # the stage convolution is the only one without a bias in the decoder: run it at the low resolution
        if b is None and x.shape[-1] % 2 == 0 and getattr(x, "_was_upsampled", False):
            return real_up(real_conv(x[:, ::2, ::2], w, None))
        return real_conv(x, w, b, stride)

    def up_mark(x):
        y = real_up(x)
        y._was_upsampled = True
        return y
    with mock.patch.object(I, "conv3x3", conv_then_upsample), mock.patch.object(I, "upsample_nearest2", up_mark):
        assert _decode_gap() > 1e-3
