"""Pins of oracle/stream.py and oracle/ssf.py against what the paper and the mathematics fix."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import ssf as F
from oracle import stream as S
from oracle import unet as U
from workloads import CONFIGS, make_weights, normal, ssf_frames, stream_inputs

DT = torch.float64
HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=DT)


def toy_eps(x, t, ctx):
    """A cheap nonlinear stand-in for the U-Net with the same signature (rows independent)."""
    rows = []
    for i in range(x.shape[0]):
        rows.append(torch.tanh(x[i] * (0.3 + 0.001 * t[i])) + 0.1 * torch.roll(x[i], 1, dims=-1) ** 2 + ctx.mean())
    return torch.stack(rows)


class Counting:
    def __init__(self, fn):
        self.fn, self.rows = fn, 0

    def __call__(self, x, t, ctx):
        self.rows += x.shape[0]
        return self.fn(x, t, ctx)


# ------------------------------------------------------------------ schedule
def test_schedule_matches_published_values():
    table = S.alphas_cumprod()
    assert table.shape == (1000,)
    with open(os.path.join(HERE, "golden", "schedule_sqrt_alpha.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 5
    for t, v, tol in rows:
        assert abs(math.sqrt(table[int(t)].item()) - float(v)) <= 1e-6 + float(tol)
    assert torch.all(table[1:] < table[:-1])
    a, b = S.ab([999, 499])
    np.testing.assert_allclose((a ** 2 + b ** 2).numpy(), 1.0, atol=1e-15)


def test_eq4_inverts_eq1():
    x0, e = _rand(4, 8, 8, seed=1), _rand(4, 8, 8, seed=2)
    for t in (999, 759, 499, 259, 1):
        a, b = S.ab([t])
        np.testing.assert_allclose(S.predict_x0(S.add_noise(x0, e, a, b), e, a, b).numpy(), x0.numpy(), atol=1e-12)


def test_cskip_cout_limits():
    assert S.c_skip_c_out(0.0) == (1.0, 0.0)
    for t in (259, 499, 759, 999):
        cs, co = S.c_skip_c_out(float(t))
        assert cs < 4e-8 and abs(co - 1.0) < 4e-8


# ------------------------------------------------------------------ guidance algebra
def test_rcfg_with_true_negative_noise_is_cfg():
    en, ep = _rand(4, 8, 8, seed=3), _rand(4, 8, 8, seed=4)
    for g in (0.0, 1.0, 1.2, 7.5):
        np.testing.assert_allclose(S.rcfg(en, ep, g, 1.0).numpy(), S.cfg(en, ep, g).numpy(), atol=1e-14)


def test_gamma_one_returns_conditional_noise():
    ev, ep = _rand(4, 8, 8, seed=5), _rand(4, 8, 8, seed=6)
    for d in (0.0, 0.5, 1.0):
        np.testing.assert_allclose(S.rcfg(ev, ep, 1.0, d).numpy(), ep.numpy(), atol=1e-14)
    np.testing.assert_allclose(S.cfg(ev, ep, 1.0).numpy(), ep.numpy(), atol=1e-14)


def test_cfg_known_numbers():
    # eps_neg = 1, eps_pos = 3, gamma = 1.5  ->  1 + 1.5 * 2 = 4 ; R-CFG with delta = 0.5: 0.5 + 1.5 * 2.5 = 4.25
    one, three = torch.ones(1, dtype=DT), 3 * torch.ones(1, dtype=DT)
    assert S.cfg(one, three, 1.5).item() == 4.0
    assert S.rcfg(one, three, 1.5, 0.5).item() == 4.25


def test_virtual_noise_at_slot0_identities():
    x0, n0, en = _rand(4, 8, 8, seed=7), _rand(4, 8, 8, seed=8), _rand(4, 8, 8, seed=9)
    a, b = S.ab([999])
    x = S.add_noise(x0, n0, a, b)
    # self-negative: Eq. 1 substituted into Eq. 5 returns the injected noise
    np.testing.assert_allclose(S.virtual_residual_noise(x, x0, a, b).numpy(), n0.numpy(), atol=1e-12)
    # onetime-negative: Eq. 7 substituted into Eq. 5 returns the true negative noise
    ref = S.predict_x0(x, en, a, b)
    np.testing.assert_allclose(S.virtual_residual_noise(x, ref, a, b).numpy(), en.numpy(), atol=1e-11)


# ------------------------------------------------------------------ Stream Batch
def _run_stream(eps_fn, ts, mode, gamma, delta, frames, S_=1, sched="lcm", seed=50):
    n = len(ts)
    x0 = _rand(frames, S_, 4, 8, 8, seed=seed)
    noise = _rand(n, S_, 4, 8, 8, seed=seed + 1)
    ctx, neg = _rand(8, 64, seed=seed + 2), _rand(8, 64, seed=seed + 3)
    sb = S.StreamBatch(eps_fn, ts, noise, mode, gamma, delta, sched)
    outs = [sb.step(x0[k], ctx, neg) for k in range(frames)]
    return x0, noise, ctx, neg, outs


@pytest.mark.parametrize("mode", [S.MODE_NONE, S.MODE_CFG, S.MODE_SELF, S.MODE_ONETIME])
@pytest.mark.parametrize("ts", [(999,), (999, 499), (999, 759, 499, 259)])
@pytest.mark.parametrize("sched", ["lcm", "ddim", "lcm_exact"])
def test_stream_batch_equals_sequential(mode, ts, sched):
    n, frames, ns = len(ts), 7, 2
    x0, noise, ctx, neg, outs = _run_stream(toy_eps, ts, mode, 1.3, 0.8, frames, ns, sched)
    for k, (out, valid) in enumerate(outs):
        assert valid == (k >= n - 1)
        if not valid:
            continue
        f = k - (n - 1)                       # the frame given n-1 calls earlier comes out now
        for s in range(ns):
            want = S.sequential_denoise(toy_eps, x0[f, s], ts, noise[:, s], ctx, neg, mode, 1.3, 0.8, sched)
            np.testing.assert_allclose(out[s].numpy(), want.numpy(), rtol=0, atol=1e-9)


def test_stream_batch_equals_sequential_with_the_real_unet():
    cfg = CONFIGS[1]
    shape = U.UNetShape.from_dict(cfg["unet"])
    net = U.UNet(shape, make_weights(U.manifest(shape), cfg["seeds"]["weights"], cfg["init"], False))
    inp = stream_inputs(cfg, 4)
    sb = S.StreamBatch(net, cfg["timesteps"], inp["noise"], cfg["cfg_mode"], cfg["gamma"], cfg["delta"])
    ctx = torch.as_tensor(inp["context"])
    outs = [sb.step(inp["x0"][k], ctx) for k in range(4)]
    for k in range(1, 4):
        want = S.sequential_denoise(net, inp["x0"][k - 1, 0], cfg["timesteps"], inp["noise"][:, 0], ctx, None,
                                    cfg["cfg_mode"], cfg["gamma"], cfg["delta"])
        assert outs[k][1]
        np.testing.assert_allclose(outs[k][0][0].numpy(), want.numpy(), rtol=0, atol=1e-10)


@pytest.mark.parametrize("mode,per_frame", [(S.MODE_NONE, lambda n: n), (S.MODE_SELF, lambda n: n),
                                            (S.MODE_ONETIME, lambda n: n + 1), (S.MODE_CFG, lambda n: 2 * n)])
def test_unet_evaluation_counts(mode, per_frame):
    for ts in [(999,), (999, 499, 259)]:
        fn = Counting(toy_eps)
        _run_stream(fn, ts, mode, 1.2, 1.0, 5)
        assert fn.rows == 5 * per_frame(len(ts))


def test_ideal_denoiser_returns_the_input_frame():
    # a denoiser that returns exactly the cached noise of the slot's step makes Eq. 4 undo Eq. 1 at every slot
    ts = (999, 759, 499, 259)
    noise = _rand(4, 1, 4, 8, 8, seed=60)
    x0 = _rand(9, 1, 4, 8, 8, seed=61)
    lookup = {t: noise[i, 0] for i, t in enumerate(ts)}

    def ideal(x, t, ctx):
        return torch.stack([lookup[int(v)] for v in t])

    for mode in (S.MODE_NONE, S.MODE_SELF):
        sb = S.StreamBatch(ideal, ts, noise, mode, 1.5, 1.0)
        for k in range(9):
            out, valid = sb.step(x0[k], None)
            if valid:
                np.testing.assert_allclose(out[0].numpy(), x0[k - 3, 0].numpy(), atol=1e-10)


def test_onetime_negative_single_step_is_full_cfg():
    ts = (999,)
    _, _, _, _, a = _run_stream(toy_eps, ts, S.MODE_ONETIME, 1.7, 1.0, 3)
    _, _, _, _, b = _run_stream(toy_eps, ts, S.MODE_CFG, 1.7, 1.0, 3)
    for (oa, _), (ob, _) in zip(a, b):
        np.testing.assert_allclose(oa.numpy(), ob.numpy(), atol=1e-10)


def test_self_negative_single_step_known_form():
    # n = 1, self-negative: eps_v = noise[0], so eps_cfg = d*n0 + g*(E - d*n0) and x0_hat follows Eq. 4 directly
    ts, g, d = (999,), 1.4, 0.6
    x0, noise, ctx, neg, outs = _run_stream(toy_eps, ts, S.MODE_SELF, g, d, 1)
    a, b = S.ab(ts)
    x = a * x0[0, 0] + b * noise[0, 0]
    e = toy_eps(x[None], [999], ctx)[0]
    want = (x - b * (d * noise[0, 0] + g * (e - d * noise[0, 0]))) / a
    np.testing.assert_allclose(outs[0][0][0].numpy(), want.numpy(), atol=1e-9)


def test_streams_do_not_interact():
    ts = (999, 499)
    x0, noise, ctx, neg, both = _run_stream(toy_eps, ts, S.MODE_SELF, 1.2, 1.0, 4, 2)
    sb = S.StreamBatch(toy_eps, ts, noise[:, 1:2], S.MODE_SELF, 1.2, 1.0)
    for k in range(4):
        out, _ = sb.step(x0[k, 1:2], ctx)
        assert torch.equal(out[0], both[k][0][1])


# ------------------------------------------------------------------ SSF
def test_ssf_integer_sums_match_python_ints():
    rng = np.random.default_rng(3)
    f, r = rng.integers(0, 256, (5, 7, 3), dtype=np.uint8), rng.integers(0, 256, (5, 7, 3), dtype=np.uint8)
    d = sum(int(a) * int(b) for a, b in zip(f.reshape(-1), r.reshape(-1)))
    nt = sum(int(a) ** 2 for a in f.reshape(-1))
    nr = sum(int(b) ** 2 for b in r.reshape(-1))
    assert F.sums(f, r) == (d, nt, nr)
    full = np.full((512, 512, 3), 255, np.uint8)        # largest possible sums stay exact
    assert F.sums(full, full) == (255 * 255 * 786432,) * 3


def test_ssf_special_cases():
    rng = np.random.default_rng(4)
    f = rng.integers(0, 256, (16, 16, 3), dtype=np.uint8)
    d, nt, nr = F.sums(f, f)
    assert F.cosine(d, nt, nr) == 1.0 and F.skip_probability(1.0, 0.98) == 1.0
    a = np.zeros((2, 2, 3), np.uint8); a[0] = 9
    b = np.zeros((2, 2, 3), np.uint8); b[1] = 7
    assert F.cosine(*F.sums(a, b)) == 0.0 and F.skip_probability(0.0, 0.98) == 0.0
    # Eq. 9 by hand: (0.99 - 0.98) / 0.02 = 0.5
    assert abs(F.skip_probability(0.99, 0.98) - 0.5) < 1e-12
    assert F.skip_probability(0.5, 0.98) == 0.0
    assert F.skip_probability(1.0, 1.0) == 0.0
    # 3-4-5: cos((3,4),(4,3)) = 24/25
    assert abs(F.cosine(24, 25, 25) - 0.96) < 1e-15
    ps = [F.skip_probability(s, 0.9) for s in np.linspace(0, 1, 101)]
    assert all(0 <= p <= 1 for p in ps) and all(q >= p for p, q in zip(ps, ps[1:]))


def test_ssf_eta_one_never_skips_and_frozen_input_skips():
    frames = list(ssf_frames(6000, 40, 32, 32))
    flt = F.Filter(1.0, 7000)
    assert not any(flt(f, k)[0] for k, f in enumerate(frames))
    flt = F.Filter(0.98, 7000)
    res = [flt(frames[0], k) for k in range(20)]
    assert res[0] == (False, 0.0)                       # first frame: no reference yet
    assert all(skip and p == 1.0 for skip, p in res[1:])


def test_ssf_reference_only_moves_on_pass():
    frames = list(ssf_frames(6000, 60, 32, 32))
    flt = F.Filter(0.98, 7000)
    ref = None
    seen = set()
    for k, f in enumerate(frames):
        skip, p = flt(f, k)
        seen.add("skip" if skip else "pass")
        if 0 < p < 1:
            seen.add("band")
        if not skip:
            ref = f
        assert np.array_equal(flt.ref, ref)
    assert seen == {"skip", "pass", "band"}


def test_ssf_uniform_draws():
    # SplitMix64 reference outputs for seed 0 (first three values of the published generator)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    got = [F.splitmix64_mix((k + 1) * 0x9E3779B97F4A7C15) for k in range(3)]
    assert got == want
    us = np.array([F.uniform(7000, k) for k in range(100000)])
    assert us.min() >= 0 and us.max() < 1
    for p in (0.1, 0.46, 0.89):
        rate = (us < p).mean()
        assert abs(rate - p) < 3 * math.sqrt(p * (1 - p) / len(us)) + 1e-3


# ------------------------------------------------------------------ exact consistency parameterisation
def test_exact_parameterisation_known_values_and_boundary():
    # appendix: c_skip = sd^2 / ((s tau)^2 + sd^2), c_out = s tau / sqrt(sd^2 + (s tau)^2) with sd = 0.5, s = 10
    cs, co = S.c_skip_c_out(0)
    assert (cs, co) == (1.0, 0.0)                          # boundary condition f(x, 0) = x
    cs, co = S.c_skip_c_out(1)
    assert abs(cs - 0.25 / 100.25) < 1e-15 and abs(co - 10.0 / 100.25 ** 0.5) < 1e-15
    cs, co = S.c_skip_c_out(259)
    assert cs < 4e-8 and 1 - co < 2e-8                     # the (0, 1) constants the paper uses are exact to fp32


def test_exact_parameterisation_is_the_shortcut_at_the_papers_timesteps_and_the_identity_at_zero():
    ts = (999, 759, 499, 259)
    _, _, _, _, a = _run_stream(toy_eps, ts, S.MODE_SELF, 1.2, 1.0, 6, 1, "lcm")
    _, _, _, _, b = _run_stream(toy_eps, ts, S.MODE_SELF, 1.2, 1.0, 6, 1, "lcm_exact")
    for (oa, va), (ob, vb) in zip(a, b):
        assert va == vb
        if va:
            assert 0 < (oa - ob).abs().max() <= 1e-6 * oa.abs().max()
    # a last step at tau = 0 hands its input latent through unchanged: x0_hat = 1 * x + 0 * (...)
    ts0 = (500, 0)
    x0, noise, ctx, neg, outs = _run_stream(toy_eps, ts0, S.MODE_NONE, 1.0, 1.0, 4, 1, "lcm_exact")
    a_, b_ = S.ab(ts0)
    for k in range(1, 4):
        f = k - 1
        x = a_[0] * x0[f, 0] + b_[0] * noise[0, 0]
        e = toy_eps(x[None], [500], ctx)[0]
        cs, co = S.c_skip_c_out(500)
        x_at_0 = a_[1] * (cs * x + co * (x - b_[0] * e) / a_[0]) + b_[1] * noise[1, 0]
        np.testing.assert_allclose(outs[k][0][0].numpy(), x_at_0.numpy(), rtol=0, atol=1e-12)


# ------------------------------------------------------------------ hard-threshold filter and run statistics
def test_hard_threshold_is_the_sign_of_eq9():
    from oracle import ssf as F
    rng = np.random.default_rng(5)
    for _ in range(200):
        a = rng.integers(0, 256, size=(6, 5, 3), dtype=np.uint8)
        b = np.clip(a.astype(np.int64) + rng.integers(-40, 41, size=a.shape), 0, 255).astype(np.uint8)
        eta = float(rng.uniform(0.8, 1.0))
        f = F.Filter(eta, 1, hard=True)
        assert f(a, 0) == (False, 0.0)                       # no reference yet: never skipped
        skip, s_c = f(b, 1)
        d, nt, nr = F.sums(b, a)
        assert s_c == F.cosine(d, nt, nr)
        assert skip == (F.skip_probability(s_c, eta) > 0.0)
    assert F.Filter(1.0, 1, hard=True)(a, 0)[0] is False and not F.Filter(1.0, 1, hard=True)(a, 1)[0]


def test_hard_threshold_sticks_where_the_sampled_filter_moves_on():
    # a scene that drifts slowly away from the first frame: every frame stays within eta of the FIRST one, so the
    # hard threshold never lets a frame through again, while Eq. 9 lets frames through with probability 1 - P
    from oracle import ssf as F
    base = np.full((8, 8, 3), 128, dtype=np.uint8)
    frames = []
    for k in range(400):
        f = base.copy()
        f[0, 0, 0] = 128 + (k % 100)                         # tiny change, similarity stays > 0.999
        frames.append(f)
    hard, soft = F.Filter(0.98, 9, hard=True), F.Filter(0.98, 9)
    hs = F.run_statistics([hard(f, k)[0] for k, f in enumerate(frames)])
    ss = F.run_statistics([soft(f, k)[0] for k, f in enumerate(frames)])
    assert hs == {"frames": 400, "processed": 1, "duty_cycle": 1 / 400, "longest_skip_run": 399}
    # with S_C = 1 - O(1e-6), P is about 0.9999: the sampled filter is nearly as sparse here, but a scene at
    # S_C = 0.99 (P = 0.5) must come through about half the time
    frames2 = []
    rng = np.random.default_rng(3)
    ref = rng.integers(0, 256, size=(16, 16, 3), dtype=np.uint8)
    for k in range(2000):
        frames2.append(ref if k % 2 == 0 else np.clip(ref.astype(np.int64) + rng.integers(-36, 37, size=ref.shape), 0, 255).astype(np.uint8))
    soft = F.Filter(0.98, 11)
    sk, ps = zip(*[soft(f, k) for k, f in enumerate(frames2)])
    expect = sum(1.0 - p for p in ps)                        # expected number of processed frames given the P's seen
    var = sum(p * (1.0 - p) for p in ps)
    assert abs((len(sk) - sum(sk)) - expect) <= 5.0 * max(var, 1.0) ** 0.5
    assert F.run_statistics(sk)["duty_cycle"] > hs["duty_cycle"]


def test_run_statistics_known_cases():
    from oracle import ssf as F
    assert F.run_statistics([]) == {"frames": 0, "processed": 0, "duty_cycle": 0.0, "longest_skip_run": 0}
    assert F.run_statistics([False, True, True, False, True]) == {"frames": 5, "processed": 2, "duty_cycle": 0.4,
                                                                  "longest_skip_run": 2}
