"""Oracle of the Stream Batch step: noise-in, batched denoising at staggered timesteps,
guidance (none / CFG / R-CFG self-negative / R-CFG onetime-negative), LCM update, queue shift.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  float64, the paper's notation:
  a_i = sqrt(alpha_{tau_i}),  b_i = sqrt(beta_{tau_i}),  beta = 1 - alpha  (Eq. 1: alpha scales the signal).

Readings of points the paper leaves open (each also listed in the design notes):
  * alpha table: cumulative product of 1 - beta_t with beta_t = linspace(sqrt(.00085), sqrt(.012), 1000)^2,
    the scaled-linear schedule of the latent-diffusion nets the paper runs.
  * c_skip = 0, c_out = 1 (the constants the paper says it uses, Sec. 3.3 and the appendix on pre-computation).
  * next latent: re-noise x0_hat to tau_{i+1} with the cached noise of step i+1 (appendix, pre-computation);
    scheduler 'ddim' uses the guided eps instead of cached noise.
  * scheduler 'lcm_exact': the consistency parameterisation of the appendix evaluated instead of replaced by
    (0, 1): x0_hat = c_skip(tau_i) x_i + c_out(tau_i) (x_i - b_i eps)/a_i, with sigma_data = 0.5, s = 10 and the
    c_out that has the limits the text states (see c_skip_c_out); at tau = 0 this is the boundary condition
    x0_hat = x.  Eq. 5 (virtual residual noise) is left as the paper derives it, under (0, 1).
  * the reference latent of Eq. 5 travels with its frame through the queue.
  * onetime-negative: Eq. 5 is applied at every slot including 0, with the reference of Eq. 7.
  * the queue starts at zero; the first n-1 outputs are flagged invalid.
"""
from __future__ import annotations

from typing import Callable, Optional, Sequence, Tuple

import torch

DT = torch.float64

MODE_NONE, MODE_CFG, MODE_SELF, MODE_ONETIME = 0, 1, 2, 3


def alphas_cumprod() -> torch.Tensor:
    betas = torch.linspace(0.00085 ** 0.5, 0.012 ** 0.5, 1000, dtype=DT) ** 2
    return torch.cumprod(1.0 - betas, dim=0)


def ab(timesteps: Sequence[int], table: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    table = alphas_cumprod() if table is None else table.to(DT)
    al = table[list(timesteps)]
    return torch.sqrt(al), torch.sqrt(1.0 - al)


def add_noise(x0, eps, a, b):
    """Eq. 1."""
    return a * x0 + b * eps


def predict_x0(x, eps, a, b):
    """Eq. 4 with c_skip = 0, c_out = 1."""
    return (x - b * eps) / a


def virtual_residual_noise(x, ref, a, b):
    """Eq. 5."""
    return (x - a * ref) / b


def cfg(eps_neg, eps_pos, gamma):
    """Eq. 2."""
    return eps_neg + gamma * (eps_pos - eps_neg)


def rcfg(eps_virtual, eps_pos, gamma, delta):
    """Eq. 6."""
    return delta * eps_virtual + gamma * (eps_pos - delta * eps_virtual)


def c_skip_c_out(tau: float, sigma_data: float = 0.5, s: float = 10.0) -> Tuple[float, float]:
    """LCM boundary functions (appendix).  The printed c_out carries a stray sigma_data in the numerator that
    contradicts the limits stated beside it (c_out -> 1); this is the form that has those limits."""
    st = s * tau
    return sigma_data ** 2 / (st ** 2 + sigma_data ** 2), st / (st ** 2 + sigma_data ** 2) ** 0.5


EpsFn = Callable[[torch.Tensor, Sequence[int], torch.Tensor], torch.Tensor]


class StreamBatch:
    """The rolling queue of Sec. 3.1: one call = one frame in, one frame out, every queued frame one step on."""

    def __init__(self, eps_fn: EpsFn, timesteps: Sequence[int], noise, mode: int = MODE_NONE,
                 gamma: float = 1.0, delta: float = 1.0, scheduler: str = "lcm", table=None):
        self.eps_fn = eps_fn
        self.t = [int(v) for v in timesteps]
        self.n = len(self.t)
        self.noise = torch.as_tensor(noise).to(DT)            # [n, S, C, H, W]
        assert self.noise.shape[0] == self.n
        self.S = self.noise.shape[1]
        self.mode, self.gamma, self.delta, self.scheduler = mode, float(gamma), float(delta), scheduler
        self.a, self.b = ab(self.t, table)
        lat = self.noise.shape[2:]
        self.q = torch.zeros((self.S, max(self.n - 1, 0)) + tuple(lat), dtype=DT)
        self.r = torch.zeros_like(self.q)
        self.calls = 0

    def step(self, x0_in, ctx, neg_ctx=None):
        x0_in = torch.as_tensor(x0_in).to(DT)
        n, a, b = self.n, self.a, self.b
        out = torch.empty_like(x0_in)
        for s in range(self.S):
            # noise-in (Eq. 1) and batch assembly (Fig. 3)
            x = [add_noise(x0_in[s], self.noise[0, s], a[0], b[0])] + [self.q[s, i - 1].clone() for i in range(1, n)]
            ref = [None] + [self.r[s, i - 1].clone() for i in range(1, n)]
            X = torch.stack(x)
            E = self.eps_fn(X, self.t, ctx)
            if self.mode == MODE_CFG:
                N = self.eps_fn(X, self.t, neg_ctx)
            if self.mode == MODE_SELF:
                ref[0] = x0_in[s]
            elif self.mode == MODE_ONETIME:
                En = self.eps_fn(X[:1], self.t[:1], neg_ctx)[0]
                ref[0] = predict_x0(x[0], En, a[0], b[0])                     # Eq. 7
            for i in range(n):
                if self.mode == MODE_NONE:
                    G = E[i]
                elif self.mode == MODE_CFG:
                    G = cfg(N[i], E[i], self.gamma)
                else:
                    G = rcfg(virtual_residual_noise(x[i], ref[i], a[i], b[i]), E[i], self.gamma, self.delta)
                X0 = predict_x0(x[i], G, a[i], b[i])
                if self.scheduler == "lcm_exact":        # f = c_skip x + c_out F of the appendix, not its (0, 1) shortcut
                    cs, co = c_skip_c_out(self.t[i])
                    X0 = cs * x[i] + co * X0
                if i < n - 1:
                    nxt = G if self.scheduler == "ddim" else self.noise[i + 1, s]
                    self.q[s, i] = add_noise(X0, nxt, a[i + 1], b[i + 1])
                    if ref[i] is not None:
                        self.r[s, i] = ref[i]
                else:
                    out[s] = X0
        valid = self.calls >= n - 1
        self.calls += 1
        return out, valid


def sequential_denoise(eps_fn: EpsFn, x0, timesteps: Sequence[int], noise, ctx, neg_ctx=None, mode: int = MODE_NONE,
                       gamma: float = 1.0, delta: float = 1.0, scheduler: str = "lcm", table=None):
    """Conventional denoising of ONE frame: n U-Net passes one after the other (the loop Stream Batch replaces).

    x0 [C,H,W]; noise [n,C,H,W] is the same per-step cache the stream uses.
    """
    x0 = torch.as_tensor(x0).to(DT)
    noise = torch.as_tensor(noise).to(DT)
    t = [int(v) for v in timesteps]
    a, b = ab(t, table)
    x = a[0] * x0 + b[0] * noise[0]
    ref = None
    for i in range(len(t)):
        e = eps_fn(x[None], [t[i]], ctx)[0]
        if mode == MODE_CFG:
            en = eps_fn(x[None], [t[i]], neg_ctx)[0]
            g = en + gamma * (e - en)
        elif mode in (MODE_SELF, MODE_ONETIME):
            if i == 0:
                if mode == MODE_SELF:
                    ref = x0
                else:
                    en = eps_fn(x[None], [t[0]], neg_ctx)[0]
                    ref = (x - b[0] * en) / a[0]
            ev = (x - a[i] * ref) / b[i]
            g = delta * ev + gamma * (e - delta * ev)
        else:
            g = e
        x0_hat = (x - b[i] * g) / a[i]
        if scheduler == "lcm_exact":
            cs, co = c_skip_c_out(t[i])
            x0_hat = cs * x + co * x0_hat
        if i + 1 < len(t):
            x = a[i + 1] * x0_hat + b[i + 1] * (g if scheduler == "ddim" else noise[i + 1])
    return x0_hat
