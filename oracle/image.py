"""Oracle of the latent <-> image stage around the U-Net: a tiny convolutional autoencoder.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's appendix only names the autoencoder it wraps around the denoiser (a tiny one, chosen for speed) and
gives neither its layers nor anything to check them against.  This file is the definition this build uses, of
the shape such tiny autoencoders have - plain 3x3 convolutions of one width, ReLU, three 2x stages - written
out with plain PyTorch CPU ops in float64, one image at a time:

  Block(x)   = ReLU( conv_c( ReLU( conv_b( ReLU( conv_a(x) ) ) ) ) + x )            (3x3, pad 1, with bias)
  encoder    : u8 image [H,W,3] / 255 -> conv3x3(3 -> w) -> Block
               -> 3 x [ conv3x3 stride 2 (w -> w, no bias) -> Block -> Block -> Block ] -> conv3x3(w -> 4)
               = latent [4, H/8, W/8]
  decoder    : z = 3 tanh(latent / 3) -> ReLU(conv3x3(4 -> w))
               -> 3 x [ Block -> Block -> Block -> nearest 2x -> conv3x3(w -> w, no bias) ] -> Block
               -> conv3x3(w -> 3) -> clamp to [0,1] = image [3, 8h, 8w];  u8 image = round(255 image), HWC

w = 64.  The weights are random (no trained autoencoder is available here), so the stage is checked as arithmetic,
not as an autoencoder: decode(encode(x)) is not close to x.
"""
from __future__ import annotations

import math
from typing import Dict, List

import numpy as np
import torch
import torch.nn.functional as F

DT = torch.float64
LATENT_CHANNELS = 4


def _block_entries(p: str, w: int) -> List[tuple]:
    e = []
    for c in "abc":
        e += [(f"{p}.{c}.w", (w, w, 3, 3), "weight"), (f"{p}.{c}.b", (w,), "bias")]
    return e


def manifest(width: int = 64) -> List[tuple]:
    """(name, shape, kind) of every tensor, encoder first, in blob order."""
    w = width
    m = [("enc.in.w", (w, 3, 3, 3), "weight"), ("enc.in.b", (w,), "bias")]
    m += _block_entries("enc.0.block.0", w)
    for s in (1, 2, 3):
        m += [(f"enc.{s}.down.w", (w, w, 3, 3), "weight")]
        for j in range(3):
            m += _block_entries(f"enc.{s}.block.{j}", w)
    m += [("enc.out.w", (LATENT_CHANNELS, w, 3, 3), "weight"), ("enc.out.b", (LATENT_CHANNELS,), "bias")]
    m += [("dec.in.w", (w, LATENT_CHANNELS, 3, 3), "weight"), ("dec.in.b", (w,), "bias")]
    for s in (0, 1, 2):
        for j in range(3):
            m += _block_entries(f"dec.{s}.block.{j}", w)
        m += [(f"dec.{s}.up.w", (w, w, 3, 3), "weight")]
    m += _block_entries("dec.3.block.0", w)
    m += [("dec.out.w", (3, w, 3, 3), "weight"), ("dec.out.b", (3,), "bias")]
    return m


def param_count(width: int = 64) -> int:
    return sum(math.prod(s) for _, s, _ in manifest(width))


def unpack(blob, width: int = 64) -> Dict[str, torch.Tensor]:
    flat = torch.as_tensor(blob).reshape(-1)
    out, off = {}, 0
    for name, shape, _ in manifest(width):
        n = math.prod(shape)
        out[name] = flat[off:off + n].reshape(shape).to(DT)
        off += n
    if off != flat.numel():
        raise ValueError(f"blob has {flat.numel()} values, manifest needs {off}")
    return out


def conv3x3(x: torch.Tensor, w: torch.Tensor, b=None, stride: int = 1) -> torch.Tensor:
    """y[o,y,x] = b[o] + sum_{c,i,j} w[o,c,i,j] x[c, y*stride+i-1, x*stride+j-1], zero outside the image."""
    return F.conv2d(x[None], w, b, stride=stride, padding=1)[0]


def relu(x: torch.Tensor) -> torch.Tensor:
    return torch.clamp(x, min=0.0)


def upsample_nearest2(x: torch.Tensor) -> torch.Tensor:
    return x.repeat_interleave(2, dim=1).repeat_interleave(2, dim=2)


def block(P, p: str, x: torch.Tensor) -> torch.Tensor:
    h = relu(conv3x3(x, P[p + ".a.w"], P[p + ".a.b"]))
    h = relu(conv3x3(h, P[p + ".b.w"], P[p + ".b.b"]))
    h = conv3x3(h, P[p + ".c.w"], P[p + ".c.b"])
    return relu(h + x)


def encode(P, image_u8: np.ndarray) -> torch.Tensor:
    """u8 image [H,W,3] (H, W multiples of 8) -> latent [4, H/8, W/8]."""
    x = torch.as_tensor(np.ascontiguousarray(image_u8)).to(DT).permute(2, 0, 1) / 255.0
    x = conv3x3(x, P["enc.in.w"], P["enc.in.b"])
    x = block(P, "enc.0.block.0", x)
    for s in (1, 2, 3):
        x = conv3x3(x, P[f"enc.{s}.down.w"], None, stride=2)
        for j in range(3):
            x = block(P, f"enc.{s}.block.{j}", x)
    return conv3x3(x, P["enc.out.w"], P["enc.out.b"])


def decode(P, latent: torch.Tensor) -> torch.Tensor:
    """latent [4,h,w] -> image [3, 8h, 8w] with values in [0,1]."""
    x = 3.0 * torch.tanh(latent.to(DT) / 3.0)
    x = relu(conv3x3(x, P["dec.in.w"], P["dec.in.b"]))
    for s in (0, 1, 2):
        for j in range(3):
            x = block(P, f"dec.{s}.block.{j}", x)
        x = conv3x3(upsample_nearest2(x), P[f"dec.{s}.up.w"], None)
    x = block(P, "dec.3.block.0", x)
    return torch.clamp(conv3x3(x, P["dec.out.w"], P["dec.out.b"]), 0.0, 1.0)


def to_u8(image: torch.Tensor) -> np.ndarray:
    """[3,H,W] in [0,1] -> u8 [H,W,3], round half to even (values are compared at +-1 level where a device rounds a
    lower-precision image)."""
    return torch.round(image * 255.0).to(torch.uint8).permute(1, 2, 0).contiguous().numpy()
