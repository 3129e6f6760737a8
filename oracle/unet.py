"""Oracle U-Net: eps = eps_theta(x, tau, c), the black box of Sec. 3.1 of the paper.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper never describes the network; it is the standard latent-diffusion U-Net whose
shape the workloads parameterise.  This file is that definition written out with plain
PyTorch CPU ops in float64, one sample at a time (batch rows of a U-Net do not interact,
which is what makes Stream Batch exact, Sec. 3.1).

  time embedding : e = [cos(t f_j) ; sin(t f_j)], f_j = exp(-ln(1e4) j / half), half = C0/2;
                   Linear(C0,4C0) -> SiLU -> Linear(4C0,4C0)
  ResBlock       : GN(eps 1e-5) -> SiLU -> conv3x3 -> + Linear(SiLU(temb)) -> GN -> SiLU
                   -> conv3x3 -> + skip (identity, or conv1x1 when the widths differ)
  Transformer    : GN(eps 1e-6) -> proj_in -> [+SelfAttn(LN)] -> [+CrossAttn(LN, ctx)]
                   -> [+GEGLU-FF(LN)] -> proj_out -> + input;  LN eps 1e-5; q/k/v without
                   bias; softmax(q k^T / sqrt(d)) v; exact (erf) GELU
  down path      : conv_in; per level: layers x (ResBlock [, Transformer]); stride-2 conv3x3
                   except after the last level; every output goes on the skip stack
  mid            : ResBlock, Transformer, ResBlock
  up path        : per level, deepest first: (layers+1) x (concat skip -> ResBlock [, Transformer]);
                   nearest 2x + conv3x3 except at level 0
  out            : GN -> SiLU -> conv3x3

Stream Batch cross-frame attention (Sec. 3.2, the two K_Batch / V_Batch equations and the Attn equation
after them): when it is on, the rows handed to one call are one stream batch; every self-attention then
uses, for each row's queries, the keys and values of ALL rows of the call concatenated along the token
axis (softmax over n x HW keys, scale 1/sqrt(d) unchanged).  Cross-attention to the prompt, and everything
else, still treats rows independently.  The paper does not say which rows form a batch under guidance;
the reading here is "the rows of one call": the positive-prompt rows of a stream, or its negative-prompt
rows, each among themselves, and the single onetime-negative row alone.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import torch
import torch.nn.functional as F

DT = torch.float64


@dataclass(frozen=True)
class UNetShape:
    in_channels: int
    block_channels: Tuple[int, ...]
    layers_per_block: int
    attn_levels: Tuple[int, ...]
    num_heads: int          # > 0: fixed head count, head width = C / num_heads
    head_dim: int           # > 0: fixed head width, head count = C / head_dim
    mid_attention: int
    context_len: int
    context_dim: int
    norm_groups: int

    @staticmethod
    def from_dict(d: dict) -> "UNetShape":
        return UNetShape(int(d["in_channels"]), tuple(int(c) for c in d["block_channels"]),
                         int(d["layers_per_block"]), tuple(int(a) for a in d["attn_levels"]),
                         int(d["num_heads"]), int(d["head_dim"]), int(d["mid_attention"]),
                         int(d["context_len"]), int(d["context_dim"]), int(d["norm_groups"]))

    def heads(self, c: int) -> int:
        if (self.num_heads > 0) == (self.head_dim > 0):
            raise ValueError("exactly one of num_heads / head_dim must be positive")
        return self.num_heads if self.num_heads > 0 else c // self.head_dim


# ----------------------------------------------------------------------------------------
# weight manifest: (name, shape, kind) in blob order
# ----------------------------------------------------------------------------------------
def _res_entries(p: str, cin: int, cout: int, temb: int) -> List[tuple]:
    e = [(p + ".norm1.g", (cin,), "gamma"), (p + ".norm1.b", (cin,), "beta"),
         (p + ".conv1.w", (cout, cin, 3, 3), "weight"), (p + ".conv1.b", (cout,), "bias"),
         (p + ".temb.w", (cout, temb), "weight"), (p + ".temb.b", (cout,), "bias"),
         (p + ".norm2.g", (cout,), "gamma"), (p + ".norm2.b", (cout,), "beta"),
         (p + ".conv2.w", (cout, cout, 3, 3), "weight"), (p + ".conv2.b", (cout,), "bias")]
    if cin != cout:
        e += [(p + ".skip.w", (cout, cin, 1, 1), "weight"), (p + ".skip.b", (cout,), "bias")]
    return e


def _tf_entries(p: str, c: int, dctx: int) -> List[tuple]:
    return [(p + ".norm.g", (c,), "gamma"), (p + ".norm.b", (c,), "beta"),
            (p + ".proj_in.w", (c, c), "weight"), (p + ".proj_in.b", (c,), "bias"),
            (p + ".ln1.g", (c,), "gamma"), (p + ".ln1.b", (c,), "beta"),
            (p + ".attn1.q.w", (c, c), "weight"), (p + ".attn1.k.w", (c, c), "weight"),
            (p + ".attn1.v.w", (c, c), "weight"),
            (p + ".attn1.o.w", (c, c), "weight"), (p + ".attn1.o.b", (c,), "bias"),
            (p + ".ln2.g", (c,), "gamma"), (p + ".ln2.b", (c,), "beta"),
            (p + ".attn2.q.w", (c, c), "weight"), (p + ".attn2.k.w", (c, dctx), "weight"),
            (p + ".attn2.v.w", (c, dctx), "weight"),
            (p + ".attn2.o.w", (c, c), "weight"), (p + ".attn2.o.b", (c,), "bias"),
            (p + ".ln3.g", (c,), "gamma"), (p + ".ln3.b", (c,), "beta"),
            (p + ".ff.in.w", (8 * c, c), "weight"), (p + ".ff.in.b", (8 * c,), "bias"),
            (p + ".ff.out.w", (c, 4 * c), "weight"), (p + ".ff.out.b", (c,), "bias"),
            (p + ".proj_out.w", (c, c), "weight"), (p + ".proj_out.b", (c,), "bias")]


def manifest(s: UNetShape) -> List[tuple]:
    ch = s.block_channels
    c0 = ch[0]
    temb = 4 * c0
    nl = len(ch)
    m = [("time.lin1.w", (temb, c0), "weight"), ("time.lin1.b", (temb,), "bias"),
         ("time.lin2.w", (temb, temb), "weight"), ("time.lin2.b", (temb,), "bias"),
         ("conv_in.w", (c0, s.in_channels, 3, 3), "weight"), ("conv_in.b", (c0,), "bias")]
    skips = [c0]
    c = c0
    for l in range(nl):
        for j in range(s.layers_per_block):
            m += _res_entries(f"down.{l}.res.{j}", c, ch[l], temb)
            c = ch[l]
            if s.attn_levels[l]:
                m += _tf_entries(f"down.{l}.attn.{j}", c, s.context_dim)
            skips.append(c)
        if l != nl - 1:
            m += [(f"down.{l}.downsample.w", (c, c, 3, 3), "weight"), (f"down.{l}.downsample.b", (c,), "bias")]
            skips.append(c)
    m += _res_entries("mid.res.0", c, c, temb)
    if s.mid_attention:
        m += _tf_entries("mid.attn", c, s.context_dim)
    m += _res_entries("mid.res.1", c, c, temb)
    for l in reversed(range(nl)):
        for j in range(s.layers_per_block + 1):
            m += _res_entries(f"up.{l}.res.{j}", c + skips.pop(), ch[l], temb)
            c = ch[l]
            if s.attn_levels[l]:
                m += _tf_entries(f"up.{l}.attn.{j}", c, s.context_dim)
        if l != 0:
            m += [(f"up.{l}.upsample.w", (c, c, 3, 3), "weight"), (f"up.{l}.upsample.b", (c,), "bias")]
    assert not skips
    m += [("out.norm.g", (c,), "gamma"), ("out.norm.b", (c,), "beta"),
          ("conv_out.w", (s.in_channels, c, 3, 3), "weight"), ("conv_out.b", (s.in_channels,), "bias")]
    return m


def param_count(s: UNetShape) -> int:
    return sum(math.prod(sh) for _, sh, _ in manifest(s))


def unpack(s: UNetShape, blob) -> Dict[str, torch.Tensor]:
    """Split a flat float32 blob (manifest order) into named float64 tensors."""
    flat = torch.as_tensor(blob).reshape(-1)
    out, off = {}, 0
    for name, shape, _ in manifest(s):
        n = math.prod(shape)
        out[name] = flat[off:off + n].reshape(shape).to(DT)
        off += n
    if off != flat.numel():
        raise ValueError(f"blob has {flat.numel()} values, manifest needs {off}")
    return out


# ----------------------------------------------------------------------------------------
# ops, each the textbook definition.  x: [C,H,W] feature maps, tokens: [T,C].
# ----------------------------------------------------------------------------------------
def conv2d(x: torch.Tensor, w: torch.Tensor, b: torch.Tensor, stride: int = 1) -> torch.Tensor:
    """y[o,y,x] = b[o] + sum_{c,i,j} w[o,c,i,j] x[c, y*stride+i-p, x*stride+j-p], zero padded, p = k//2."""
    return F.conv2d(x[None], w, b, stride=stride, padding=w.shape[-1] // 2)[0]


def group_norm(x: torch.Tensor, groups: int, g: torch.Tensor, b: torch.Tensor, eps: float) -> torch.Tensor:
    """Per group of C/groups channels: (x - mean) / sqrt(var + eps), biased variance over the group's C/G*H*W values."""
    c, h, w = x.shape
    xg = x.reshape(groups, -1)
    mu = xg.mean(dim=1, keepdim=True)
    var = ((xg - mu) ** 2).mean(dim=1, keepdim=True)
    y = ((xg - mu) / torch.sqrt(var + eps)).reshape(c, h, w)
    return y * g[:, None, None] + b[:, None, None]


def layer_norm(x: torch.Tensor, g: torch.Tensor, b: torch.Tensor, eps: float = 1e-5) -> torch.Tensor:
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + eps) * g + b


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


def gelu_erf(x: torch.Tensor) -> torch.Tensor:
    return 0.5 * x * (1.0 + torch.erf(x / math.sqrt(2.0)))


def attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, heads: int) -> torch.Tensor:
    """q [Tq,C], k,v [Tk,C]; per head h over columns [h d, (h+1) d): softmax(q k^T / sqrt(d)) v."""
    tq, c = q.shape
    d = c // heads
    out = torch.empty_like(q)
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        s = q[:, sl] @ k[:, sl].T / math.sqrt(d)
        s = s - s.max(dim=1, keepdim=True).values
        p = torch.exp(s)
        p = p / p.sum(dim=1, keepdim=True)
        out[:, sl] = p @ v[:, sl]
    return out


def time_embedding(t: int, c0: int) -> torch.Tensor:
    half = c0 // 2
    j = torch.arange(half, dtype=DT)
    f = torch.exp(-math.log(10000.0) * j / half)
    a = float(t) * f
    return torch.cat([torch.cos(a), torch.sin(a)])


def upsample_nearest2(x: torch.Tensor) -> torch.Tensor:
    return x.repeat_interleave(2, dim=1).repeat_interleave(2, dim=2)


# ----------------------------------------------------------------------------------------
# blocks
# ----------------------------------------------------------------------------------------
def _linear(x, w, b=None):
    y = x @ w.T
    return y if b is None else y + b


def res_block(P, p: str, x, temb, groups: int):
    h = conv2d(silu(group_norm(x, groups, P[p + ".norm1.g"], P[p + ".norm1.b"], 1e-5)),
               P[p + ".conv1.w"], P[p + ".conv1.b"])
    h = h + _linear(silu(temb), P[p + ".temb.w"], P[p + ".temb.b"])[:, None, None]
    h = conv2d(silu(group_norm(h, groups, P[p + ".norm2.g"], P[p + ".norm2.b"], 1e-5)),
               P[p + ".conv2.w"], P[p + ".conv2.b"])
    if (p + ".skip.w") in P:
        x = conv2d(x, P[p + ".skip.w"], P[p + ".skip.b"])
    return x + h


def transformer_rows(P, p: str, xs, ctx, heads: int, groups: int, cross_frame: bool):
    """The transformer block on a list of rows.  Only the self-attention can couple rows (cross_frame)."""
    c, hh, ww = xs[0].shape
    hs = []
    for x in xs:
        h = group_norm(x, groups, P[p + ".norm.g"], P[p + ".norm.b"], 1e-6)
        h = h.reshape(c, hh * ww).T                               # tokens [HW, C]
        hs.append(_linear(h, P[p + ".proj_in.w"], P[p + ".proj_in.b"]))
    ns = [layer_norm(h, P[p + ".ln1.g"], P[p + ".ln1.b"]) for h in hs]
    qs = [_linear(n, P[p + ".attn1.q.w"]) for n in ns]
    ks = [_linear(n, P[p + ".attn1.k.w"]) for n in ns]
    vs = [_linear(n, P[p + ".attn1.v.w"]) for n in ns]
    if cross_frame:
        k_batch, v_batch = torch.cat(ks, dim=0), torch.cat(vs, dim=0)     # K_Batch, V_Batch of Sec. 3.2
        att = [attention(q, k_batch, v_batch, heads) for q in qs]
    else:
        att = [attention(q, k, v, heads) for q, k, v in zip(qs, ks, vs)]
    out = []
    for x, h, a in zip(xs, hs, att):
        h = h + _linear(a, P[p + ".attn1.o.w"], P[p + ".attn1.o.b"])
        n = layer_norm(h, P[p + ".ln2.g"], P[p + ".ln2.b"])
        a = attention(_linear(n, P[p + ".attn2.q.w"]), _linear(ctx, P[p + ".attn2.k.w"]),
                      _linear(ctx, P[p + ".attn2.v.w"]), heads)
        h = h + _linear(a, P[p + ".attn2.o.w"], P[p + ".attn2.o.b"])
        n = layer_norm(h, P[p + ".ln3.g"], P[p + ".ln3.b"])
        u = _linear(n, P[p + ".ff.in.w"], P[p + ".ff.in.b"])
        inner = u.shape[1] // 2
        u = u[:, :inner] * gelu_erf(u[:, inner:])
        h = h + _linear(u, P[p + ".ff.out.w"], P[p + ".ff.out.b"])
        h = _linear(h, P[p + ".proj_out.w"], P[p + ".proj_out.b"])
        out.append(x + h.T.reshape(c, hh, ww))
    return out


def transformer(P, p: str, x, ctx, heads: int, groups: int):
    return transformer_rows(P, p, [x], ctx, heads, groups, False)[0]


def unet_rows(s: UNetShape, P: Dict[str, torch.Tensor], xs, ts: Sequence[int], ctx: torch.Tensor,
              cross_frame: bool = False) -> List[torch.Tensor]:
    """Rows xs[i] [C_in,H,W] at integer timesteps ts[i], ctx [L,D] shared -> predicted noise per row.
    Rows interact only through the self-attention, and only when cross_frame is set."""
    ch = s.block_channels
    nl = len(ch)
    g = s.norm_groups
    R = range(len(xs))
    ctx = ctx.to(DT)
    tembs = []
    for t in ts:
        e = time_embedding(int(t), ch[0])
        tembs.append(_linear(silu(_linear(e, P["time.lin1.w"], P["time.lin1.b"])), P["time.lin2.w"], P["time.lin2.b"]))
    hs = [conv2d(x.to(DT), P["conv_in.w"], P["conv_in.b"]) for x in xs]
    skips = [hs]
    for l in range(nl):
        for j in range(s.layers_per_block):
            hs = [res_block(P, f"down.{l}.res.{j}", hs[r], tembs[r], g) for r in R]
            if s.attn_levels[l]:
                hs = transformer_rows(P, f"down.{l}.attn.{j}", hs, ctx, s.heads(ch[l]), g, cross_frame)
            skips.append(hs)
        if l != nl - 1:
            hs = [conv2d(h, P[f"down.{l}.downsample.w"], P[f"down.{l}.downsample.b"], stride=2) for h in hs]
            skips.append(hs)
    hs = [res_block(P, "mid.res.0", hs[r], tembs[r], g) for r in R]
    if s.mid_attention:
        hs = transformer_rows(P, "mid.attn", hs, ctx, s.heads(ch[-1]), g, cross_frame)
    hs = [res_block(P, "mid.res.1", hs[r], tembs[r], g) for r in R]
    for l in reversed(range(nl)):
        for j in range(s.layers_per_block + 1):
            sk = skips.pop()
            hs = [res_block(P, f"up.{l}.res.{j}", torch.cat([hs[r], sk[r]], dim=0), tembs[r], g) for r in R]
            if s.attn_levels[l]:
                hs = transformer_rows(P, f"up.{l}.attn.{j}", hs, ctx, s.heads(ch[l]), g, cross_frame)
        if l != 0:
            hs = [conv2d(upsample_nearest2(h), P[f"up.{l}.upsample.w"], P[f"up.{l}.upsample.b"]) for h in hs]
    assert not skips
    hs = [silu(group_norm(h, g, P["out.norm.g"], P["out.norm.b"], 1e-5)) for h in hs]
    return [conv2d(h, P["conv_out.w"], P["conv_out.b"]) for h in hs]


def unet_single(s: UNetShape, P: Dict[str, torch.Tensor], x: torch.Tensor, t: int, ctx: torch.Tensor) -> torch.Tensor:
    """One sample: x [C_in,H,W], integer timestep t, ctx [L,D] -> predicted noise [C_in,H,W]."""
    return unet_rows(s, P, [x], [t], ctx, False)[0]


class UNet:
    """eps_theta with a call counter (the paper counts U-Net evaluations per frame, Sec. 3.3).
    cross_frame: the rows of one call form a stream batch for cross-frame attention (Sec. 3.2)."""

    def __init__(self, shape: UNetShape, blob, cross_frame: bool = False):
        self.shape = shape
        self.P = unpack(shape, blob)
        self.cross_frame = bool(cross_frame)
        self.evaluations = 0

    def __call__(self, x: torch.Tensor, t: Sequence[int], ctx: torch.Tensor) -> torch.Tensor:
        """x [N,C,H,W], t [N], ctx [L,D] shared by all rows -> eps [N,C,H,W]."""
        self.evaluations += x.shape[0]
        if self.cross_frame:
            return torch.stack(unet_rows(self.shape, self.P, list(x), [int(v) for v in t], ctx, True))
        return torch.stack([unet_single(self.shape, self.P, x[i], int(t[i]), ctx) for i in range(x.shape[0])])
