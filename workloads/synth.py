"""Seeded synthetic workloads (stand-ins for the paper's prompts, videos and trained nets).

Everything is drawn from numpy's Philox counter-based bit generator keyed by
(seed, crc32(name)), so any tensor can be regenerated on its own, in any order,
here or on the GPU machine.  The U-Net *shape* of each workload is a plain dict; the
oracle and the HIP library each turn it into their own weight manifest, and
`make_weights` fills whichever manifest it is handed.
"""
from __future__ import annotations

import zlib
from typing import Iterable, Iterator, Sequence

import numpy as np


def _rng(seed: int, name: str) -> np.random.Generator:
    key = np.array([np.uint64(seed), np.uint64(zlib.crc32(name.encode()))], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal(seed: int, name: str, shape: Sequence[int], std: float = 1.0) -> np.ndarray:
    """float32 N(0, std²) tensor identified by (seed, name)."""
    a = _rng(seed, name).standard_normal(size=tuple(shape), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable value (ties to even), kept as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def make_weights(manifest: Iterable, seed: int, init: str, bf16_round: bool) -> np.ndarray:
    """Fill a flat float32 blob for `manifest` = iterable of (name, shape, kind).

    kind: 'weight' (conv OIHW or linear [out,in]), 'bias', 'gamma', 'beta'.
    init 'n002' : weights and biases ~ N(0, 0.02²); gamma = 1; beta = 0.
    init 'fanin': weights ~ N(0, 1/fan_in); biases ~ N(0, 0.02²); gamma = 1; beta = 0.
    init 'fanin_affine': as 'fanin' with gamma ~ 1 + N(0, 0.2²) and beta ~ N(0, 0.1²), so that a norm's scale and
                  shift are visible in the output (folded or fused norm parameters cannot hide behind 1 and 0).
    bf16_round  : round every value to a bf16-representable float32.
    """
    manifest = list(manifest)
    total = sum(int(np.prod(s)) for _, s, _ in manifest)
    blob = np.empty(total, dtype=np.float32)
    off = 0
    for name, shape, kind in manifest:
        n = int(np.prod(shape))
        if kind == "gamma":
            blob[off:off + n] = 1.0 + normal(seed, name, (n,), 0.2) if init == "fanin_affine" else 1.0
        elif kind == "beta":
            blob[off:off + n] = normal(seed, name, (n,), 0.1) if init == "fanin_affine" else 0.0
        elif kind == "bias":
            blob[off:off + n] = normal(seed, name, (n,), 0.02)
        elif kind == "weight":
            if init == "n002":
                std = 0.02
            elif init in ("fanin", "fanin_affine"):
                std = 1.0 / float(np.sqrt(np.prod(shape[1:])))
            else:
                raise ValueError(init)
            blob[off:off + n] = normal(seed, name, (n,), std)
        else:
            raise ValueError(kind)
        off += n
    if bf16_round:
        blob = round_to_bf16(blob)
    return blob


# --------------------------------------------------------------------------------------
# workload table.  "unet" is the shape descriptor; the rest describes the stream.
# cfg_mode: 0 none, 1 full CFG, 2 R-CFG self-negative, 3 R-CFG onetime-negative.
# --------------------------------------------------------------------------------------
_SD15 = dict(in_channels=4, block_channels=(320, 640, 1280, 1280), layers_per_block=2,
             attn_levels=(1, 1, 1, 0), num_heads=8, head_dim=0, mid_attention=1,
             context_len=77, context_dim=768, norm_groups=32)
_SD21 = dict(_SD15, num_heads=0, head_dim=64, context_dim=1024)
_TINY = dict(in_channels=4, block_channels=(32, 64), layers_per_block=1, attn_levels=(0, 1),
             num_heads=0, head_dim=32, mid_attention=1, context_len=8, context_dim=64, norm_groups=8)


def _seeds(c: int) -> dict:
    return dict(weights=1000 + c, noise=2000 + c, inputs=3000 + c, context=4000 + c, neg_context=5000 + c)


CONFIGS = {
    1: dict(name="tiny-fp32", unet=_TINY, latent=(8, 8), dtype="fp32", init="n002",
            timesteps=(999, 499), n_streams=1, cfg_mode=2, gamma=1.4, delta=1.0, frames=16, seeds=_seeds(1)),
    2: dict(name="sd21-b1", unet=_SD21, latent=(64, 64), dtype="bf16", init="fanin",
            timesteps=(999,), n_streams=1, cfg_mode=0, gamma=1.0, delta=1.0, frames=256, seeds=_seeds(2)),
    3: dict(name="sd15-b4", unet=_SD15, latent=(64, 64), dtype="bf16", init="fanin",
            timesteps=(999, 759, 499, 259), n_streams=1, cfg_mode=0, gamma=1.0, delta=1.0, frames=512,
            seeds=_seeds(3)),
    4: dict(name="sd15-b4-guidance", unet=_SD15, latent=(64, 64), dtype="bf16", init="fanin",
            timesteps=(999, 759, 499, 259), n_streams=1, cfg_mode=(1, 2, 3), gamma=1.2, delta=1.0, frames=512,
            seeds=_seeds(4)),
    5: dict(name="sd15-b4x4-96", unet=_SD15, latent=(96, 96), dtype="bf16", init="fanin",
            timesteps=(999, 759, 499, 259), n_streams=4, cfg_mode=2, gamma=1.2, delta=1.0, frames=512,
            seeds=_seeds(5), ssf=dict(frames=512, h=512, w=512, eta=0.98, frame_seed=6000, draw_seed=7000)),
}

# Reduced shapes with the structure of the SD nets (4 levels, 2 ResBlocks per level, attention on the
# first three levels, skip concats with unequal halves, ragged pixel counts): sized so the CPU oracle
# finishes in seconds while every GPU kernel still spans several tiles plus a tail.
_MINI15 = dict(in_channels=4, block_channels=(64, 128, 256, 256), layers_per_block=2,
               attn_levels=(1, 1, 1, 0), num_heads=8, head_dim=0, mid_attention=1,
               context_len=13, context_dim=96, norm_groups=32)
_MINI21 = dict(_MINI15, num_heads=0, head_dim=64, context_len=77, context_dim=128)
_MINI40 = dict(in_channels=4, block_channels=(160, 320, 640), layers_per_block=1,
               attn_levels=(1, 1, 0), num_heads=4, head_dim=0, mid_attention=1,
               context_len=77, context_dim=192, norm_groups=32)

# one wide level (320 channels on 4 x 62 x 58 = 14 384 pixels, a ragged number of 64- and 128-row tiles): the shape
# class of the first level of the SD nets, which some kernels are specialised for, at a size the oracle still finishes
_WIDE320 = dict(in_channels=4, block_channels=(320, 640), layers_per_block=1,
                attn_levels=(1, 0), num_heads=8, head_dim=0, mid_attention=0,
                context_len=77, context_dim=128, norm_groups=32)

MINI_CONFIGS = {
    "wide320": dict(name="wide320", unet=_WIDE320, latent=(62, 58), init="fanin",
                    timesteps=(999, 499), n_streams=1, seeds=_seeds(14)),
    "mini15": dict(name="mini15", unet=_MINI15, latent=(24, 40), init="fanin",
                   timesteps=(999, 759, 499, 259), n_streams=1, seeds=_seeds(11)),
    "mini21": dict(name="mini21", unet=_MINI21, latent=(16, 16), init="fanin",
                   timesteps=(999, 499), n_streams=2, seeds=_seeds(12)),
    "mini40": dict(name="mini40", unet=_MINI40, latent=(20, 12), init="fanin",
                   timesteps=(999, 599, 199), n_streams=1, seeds=_seeds(13)),
}


def stream_inputs(cfg: dict, n_frames: int) -> dict:
    """Latents, contexts and the per-step noise cache of a workload, all i.i.d. N(0,1) float32."""
    u = cfg["unet"]
    h, w = cfg["latent"]
    s = cfg["n_streams"]
    n = len(cfg["timesteps"])
    sd = cfg["seeds"]
    return dict(
        x0=normal(sd["inputs"], "x0", (n_frames, s, u["in_channels"], h, w)),
        noise=normal(sd["noise"], "noise", (n, s, u["in_channels"], h, w)),
        context=normal(sd["context"], "context", (u["context_len"], u["context_dim"])),
        neg_context=normal(sd["neg_context"], "neg_context", (u["context_len"], u["context_dim"])),
    )


IMAGE_STAGE = dict(width=64, init="fanin", seeds=dict(weights=8000, images=8100, latents=8200))


def image_frames(seed: int, n_frames: int, n_streams: int, h: int, w: int) -> np.ndarray:
    """u8 [n_frames, n_streams, h, w, 3] stand-ins for camera frames: i.i.d. uniform pixels blurred 3x3 (neighbouring
    pixels correlate, as in photographs), each frame drawn on its own."""
    a = _rng(seed, f"images{h}x{w}").integers(0, 256, size=(n_frames, n_streams, h + 2, w + 2, 3)).astype(np.float32)
    b = sum(a[:, :, i:i + h, j:j + w] for i in range(3) for j in range(3)) / 9.0
    lo, hi = b.min(), b.max()
    return np.clip(np.rint((b - lo) / (hi - lo) * 255.0), 0, 255).astype(np.uint8)


def ssf_frames(seed: int, n_frames: int, h: int, w: int, static_run: int = 12, perturbed_run: int = 8,
               sigmas: Sequence[float] = (10.0, 20.0, 30.0, 60.0)) -> Iterator[np.ndarray]:
    """Synthetic u8 H×W×3 frame sequence: runs of exact repeats alternate with Gaussian-perturbed runs.

    A cycle is `static_run` identical copies of the scene base followed by `perturbed_run` frames
    clip(round(base + sigma*z)) with sigma cycling through `sigmas` (60 % static / 40 % perturbed with
    the defaults).  The base is redrawn every fourth cycle.
    """
    cycle = static_run + perturbed_run
    base = None
    for k in range(n_frames):
        c, j = divmod(k, cycle)
        if base is None or (j == 0 and c % 4 == 0):
            base = _rng(seed, f"base{c}").integers(0, 256, size=(h, w, 3), dtype=np.uint8)
        if j < static_run:
            yield base.copy()
        else:
            sigma = sigmas[(j - static_run) % len(sigmas)]
            z = _rng(seed, f"z{k}").standard_normal(size=(h, w, 3), dtype=np.float32)
            f = np.rint(base.astype(np.float32) + np.float32(sigma) * z)
            yield np.clip(f, 0, 255).astype(np.uint8)
