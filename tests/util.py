"""Helpers shared by the GPU parity tests: build an engine / an oracle net for one workload dict."""
import numpy as np
import torch

from workloads import make_weights


def rel_max(g, o):
    g, o = np.asarray(g, dtype=np.float64), np.asarray(o, dtype=np.float64)
    return float(np.abs(g - o).max() / np.abs(o).max())


def rel_l2(g, o):
    g, o = np.asarray(g, dtype=np.float64), np.asarray(o, dtype=np.float64)
    return float(np.linalg.norm(g - o) / np.linalg.norm(o))


TOL_BF16 = 2e-2       # ||g-o||_2 / ||o||_2 (the stated bf16 tolerance)
TOL_BF16_MAX = 3e-2   # max|g-o| / max|o|: a guard against a localised defect that a norm over 16 384 values absorbs


def check_bf16(g, o, what=""):
    """Both bf16 criteria on one output; prints what was observed (shown with pytest -s / -rP) and returns the pair."""
    l2, mx = rel_l2(g, o), rel_max(g, o)
    print(f"bf16 parity {what}: rel_l2 {l2:.3e} (<= {TOL_BF16:g}), max|g-o|/max|o| {mx:.3e} (<= {TOL_BF16_MAX:g})")
    assert l2 <= TOL_BF16, (what, l2)
    assert mx <= TOL_BF16_MAX, (what, mx)
    return l2, mx


def oracle_net(wl, bf16_weights, cross_frame=False):
    from oracle import unet as U
    shape = U.UNetShape.from_dict(wl["unet"])
    blob = make_weights(U.manifest(shape), wl["seeds"]["weights"], wl["init"], bf16_weights)
    return U.UNet(shape, blob, cross_frame=cross_frame)


def gpu_engine(wl, dtype, cfg_mode=0, scheduler=0, n_streams=None, timesteps=None, blob=None, cross_frame=0):
    import paper_2312_12491_amd as sd
    ts = wl["timesteps"] if timesteps is None else timesteps
    S = wl["n_streams"] if n_streams is None else n_streams
    cfg = sd.config_from_dict(wl["unet"], wl["latent"], dtype, len(ts), S, cfg_mode, scheduler, cross_frame)
    eng = sd.Engine(cfg)
    if blob is None:
        blob = make_weights(eng.manifest(), wl["seeds"]["weights"], wl["init"], dtype == "bf16")
    eng.load_weights(blob)
    return eng


def cuda(a):
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()
