"""ctypes binding of include/sdstream.h: argument marshalling only, same names as the C ABI."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libsdstream.so")

CFG_NONE, CFG_FULL, CFG_SELF, CFG_ONETIME = 0, 1, 2, 3
MAX_LEVELS = 8


class SdstreamError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sdstream error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("in_channels", C.c_int32), ("n_levels", C.c_int32), ("block_channels", C.c_int32 * MAX_LEVELS),
                ("layers_per_block", C.c_int32), ("attn_level_mask", C.c_uint32), ("num_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mid_attention", C.c_int32), ("context_len", C.c_int32),
                ("context_dim", C.c_int32), ("norm_groups", C.c_int32), ("latent_h", C.c_int32),
                ("latent_w", C.c_int32), ("dtype", C.c_int32), ("n_denoise", C.c_int32), ("n_streams", C.c_int32),
                ("cfg_mode", C.c_int32), ("scheduler", C.c_int32), ("cross_frame", C.c_int32),
                ("image_width", C.c_int32)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib = None

_SIGNATURES = {
    "sdstream_create": (C.c_int, [C.POINTER(Config), C.POINTER(C.c_void_p)]),
    "sdstream_destroy": (None, [C.c_void_p]),
    "sdstream_last_error": (C.c_char_p, [C.c_void_p]),
    "sdstream_param_count": (C.c_int64, [C.c_void_p]),
    "sdstream_manifest_size": (C.c_int32, [C.c_void_p]),
    "sdstream_manifest_entry": (C.c_int, [C.c_void_p, C.c_int32, C.c_char_p, C.c_size_t, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "sdstream_load_weights": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "sdstream_image_param_count": (C.c_int64, [C.c_void_p]),
    "sdstream_image_manifest_size": (C.c_int32, [C.c_void_p]),
    "sdstream_image_manifest_entry": (C.c_int, [C.c_void_p, C.c_int32, C.c_char_p, C.c_size_t, C.POINTER(C.c_int32),
                                                C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "sdstream_load_image_weights": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "sdstream_encode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sdstream_decode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sdstream_step_image": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_int32),
                                      C.c_float, C.c_float, C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]),
    "sdstream_set_schedule": (C.c_int, [C.c_void_p, C.c_void_p]),
    "sdstream_set_noise": (C.c_int, [C.c_void_p, C.c_void_p]),
    "sdstream_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_int32),
                                C.c_float, C.c_float, C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]),
    "sdstream_unet_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p]),
    "sdstream_max_batch": (C.c_int32, [C.c_void_p]),
    "sdstream_ssf": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_uint64, C.c_uint64,
                               C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_void_p]),
    "sdstream_ssf_decide": (C.c_int, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_double, C.c_uint64, C.c_uint64,
                                      C.POINTER(C.c_double)]),
    "sdstream_ssf_decide_hard": (C.c_int, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_double, C.POINTER(C.c_double)]),
    "sdstream_ssf_hard": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.POINTER(C.c_int32),
                                    C.POINTER(C.c_double), C.c_void_p]),
    "sdstream_ssf_run_stats": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                         C.POINTER(C.c_int64)]),
    "sdstream_ssf_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_uint64, C.c_uint64,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sdstream_reset": (C.c_int, [C.c_void_p]),
    "sdstream_flops_per_row": (C.c_double, [C.c_void_p]),
    "sdstream_mfma_ceiling": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_void_p]),
    "sdstream_profile_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "sdstream_profile_reset": (C.c_int, [C.c_void_p]),
    "sdstream_profile_read": (C.c_int32, [C.c_void_p, C.POINTER(ProfileEntry), C.c_int32]),
    "sdstream_use_graph": (C.c_int, [C.c_void_p, C.c_int32]),
}


def lib():
    """Loads libsdstream.so (built in-tree by build.py); raises if it is missing - there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2312_12491_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def config_from_dict(unet: dict, latent, dtype: str, n_denoise: int, n_streams: int, cfg_mode: int,
                     scheduler: int = 0, cross_frame: int = 0, image_width: int = 0) -> Config:
    c = Config()
    ch = list(unet["block_channels"])
    c.in_channels = unet["in_channels"]
    c.n_levels = len(ch)
    for i, v in enumerate(ch):
        c.block_channels[i] = v
    c.layers_per_block = unet["layers_per_block"]
    c.attn_level_mask = sum(1 << i for i, a in enumerate(unet["attn_levels"]) if a)
    c.num_heads, c.head_dim = unet["num_heads"], unet["head_dim"]
    c.mid_attention = unet["mid_attention"]
    c.context_len, c.context_dim = unet["context_len"], unet["context_dim"]
    c.norm_groups = unet["norm_groups"]
    c.latent_h, c.latent_w = latent
    c.dtype = {"fp32": 0, "bf16": 1}[dtype]
    c.n_denoise, c.n_streams, c.cfg_mode, c.scheduler = n_denoise, n_streams, cfg_mode, scheduler
    c.cross_frame = int(cross_frame)
    c.image_width = int(image_width)
    return c


def ssf_decide(dot: int, n_t: int, n_ref: int, eta: float, seed: int, frame_index: int):
    p = C.c_double()
    skip = lib().sdstream_ssf_decide(dot, n_t, n_ref, eta, seed, frame_index, C.byref(p))
    return bool(skip), p.value


def ssf_decide_hard(dot: int, n_t: int, n_ref: int, eta: float):
    sc = C.c_double()
    skip = lib().sdstream_ssf_decide_hard(dot, n_t, n_ref, eta, C.byref(sc))
    return bool(skip), sc.value


def ssf_static(frame, reference, height: int, width: int, eta: float, seed: int, frame_index: int, sums_out,
               skip_out, prob_out, stream: int = 0):
    """sdstream_ssf_static: torch CUDA tensors (uint8 frames; int64 [3], int32 [1], float64 [1] outputs; reference,
    sums_out and prob_out may be None).  Enqueues only; raises on a rejected call."""
    rc = lib().sdstream_ssf_static(_ptr(frame), _ptr(reference), height, width, eta, seed, frame_index,
                                   _ptr(sums_out), _ptr(skip_out), _ptr(prob_out), stream or None)
    if rc < 0:
        raise SdstreamError(rc, lib().sdstream_last_error(None).decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Engine:
    """One sdstream handle.  Tensor arguments are torch CUDA tensors (float32, contiguous) unless noted."""

    def __init__(self, cfg: Config):
        self._l = lib()
        self.cfg = cfg
        h = C.c_void_p()
        rc = self._l.sdstream_create(C.byref(cfg), C.byref(h))
        if rc != 0:
            raise SdstreamError(rc, self._l.sdstream_last_error(None).decode())
        self._h = h

    def _check(self, rc: int):
        if rc < 0:
            raise SdstreamError(rc, self._l.sdstream_last_error(self._h).decode())
        return rc

    def close(self):
        if getattr(self, "_h", None):
            self._l.sdstream_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- queries
    def param_count(self) -> int:
        return self._l.sdstream_param_count(self._h)

    def max_batch(self) -> int:
        return self._l.sdstream_max_batch(self._h)

    def flops_per_row(self) -> float:
        return self._l.sdstream_flops_per_row(self._h)

    def _manifest(self, size_fn, entry_fn):
        out = []
        kinds = {0: "weight", 1: "bias", 2: "gamma", 3: "beta"}
        name = C.create_string_buffer(128)
        shape = (C.c_int32 * 4)()
        ndim, kind = C.c_int32(), C.c_int32()
        for i in range(size_fn(self._h)):
            self._check(entry_fn(self._h, i, name, 128, shape, C.byref(ndim), C.byref(kind)))
            out.append((name.value.decode(), tuple(shape[j] for j in range(ndim.value)), kinds[kind.value]))
        return out

    def manifest(self):
        return self._manifest(self._l.sdstream_manifest_size, self._l.sdstream_manifest_entry)

    def image_manifest(self):
        return self._manifest(self._l.sdstream_image_manifest_size, self._l.sdstream_image_manifest_entry)

    def image_param_count(self) -> int:
        return self._l.sdstream_image_param_count(self._h)

    def load_image_weights(self, blob):
        """blob: contiguous float32 numpy array in image-manifest order."""
        assert blob.dtype.name == "float32" and blob.flags["C_CONTIGUOUS"]
        self._check(self._l.sdstream_load_image_weights(self._h, blob.ctypes.data, blob.nbytes))

    def encode(self, image, latent_out, stream: int = 0):
        """image: torch uint8 CUDA [S,H,W,3]; latent_out: float32 CUDA [S,4,H/8,W/8]."""
        self._check(self._l.sdstream_encode(self._h, _ptr(image), _ptr(latent_out), stream or None))

    def decode(self, latent, image_out=None, image_f32_out=None, stream: int = 0):
        self._check(self._l.sdstream_decode(self._h, _ptr(latent), _ptr(image_out), _ptr(image_f32_out), stream or None))

    def step_image(self, frame, context, neg_context, context_epoch: int, timesteps: Sequence[int], gamma: float,
                   delta: float, image_out, stream: int = 0) -> bool:
        ts = (C.c_int32 * len(timesteps))(*timesteps)
        valid = C.c_int32()
        self._check(self._l.sdstream_step_image(self._h, _ptr(frame), _ptr(context), _ptr(neg_context), context_epoch,
                                                ts, gamma, delta, _ptr(image_out), C.byref(valid), stream or None))
        return bool(valid.value)

    # ---- setup
    def load_weights(self, blob):
        """blob: contiguous float32 numpy array in manifest order."""
        assert blob.dtype.name == "float32" and blob.flags["C_CONTIGUOUS"]
        self._check(self._l.sdstream_load_weights(self._h, blob.ctypes.data, blob.nbytes))

    def set_schedule(self, alphas_cumprod=None):
        if alphas_cumprod is None:
            self._check(self._l.sdstream_set_schedule(self._h, None))
        else:
            assert alphas_cumprod.dtype.name == "float32" and alphas_cumprod.size == 1000
            self._check(self._l.sdstream_set_schedule(self._h, alphas_cumprod.ctypes.data))

    def set_noise(self, noise):
        """noise: contiguous float32 numpy array [n, S, C, H, W]."""
        assert noise.dtype.name == "float32" and noise.flags["C_CONTIGUOUS"]
        self._check(self._l.sdstream_set_noise(self._h, noise.ctypes.data))

    def reset(self):
        self._check(self._l.sdstream_reset(self._h))

    def use_graph(self, on: bool):
        self._check(self._l.sdstream_use_graph(self._h, int(on)))

    # ---- hot path
    def step(self, x0_in, context, neg_context, context_epoch: int, timesteps: Sequence[int], gamma: float,
             delta: float, out_latent, stream: int = 0) -> bool:
        ts = (C.c_int32 * len(timesteps))(*timesteps)
        valid = C.c_int32()
        self._check(self._l.sdstream_step(self._h, _ptr(x0_in), _ptr(context), _ptr(neg_context), context_epoch, ts,
                                          gamma, delta, _ptr(out_latent), C.byref(valid), stream or None))
        return bool(valid.value)

    def unet_forward(self, x, t: Sequence[int], ctx, eps_out, stream: int = 0):
        ts = (C.c_int32 * len(t))(*t)
        self._check(self._l.sdstream_unet_forward(self._h, _ptr(x), ts, _ptr(ctx), len(t), _ptr(eps_out),
                                                  stream or None))

    def ssf(self, frame, height: int, width: int, eta: float, seed: int, frame_index: int, stream: int = 0):
        """frame: torch uint8 CUDA tensor [H, W, 3].  Returns (skip, probability)."""
        skip, p = C.c_int32(), C.c_double()
        self._check(self._l.sdstream_ssf(self._h, _ptr(frame), height, width, eta, seed, frame_index, C.byref(skip),
                                         C.byref(p), stream or None))
        return bool(skip.value), p.value

    def ssf_hard(self, frame, height: int, width: int, eta: float, stream: int = 0):
        """Hard-threshold filter.  frame: torch uint8 CUDA tensor [H, W, 3].  Returns (skip, similarity)."""
        skip, sc = C.c_int32(), C.c_double()
        self._check(self._l.sdstream_ssf_hard(self._h, _ptr(frame), height, width, eta, C.byref(skip), C.byref(sc),
                                              stream or None))
        return bool(skip.value), sc.value

    def ssf_run_stats(self):
        """(frames seen, frames let through, longest run of consecutive skips) since the last reset."""
        f, p, l = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self._l.sdstream_ssf_run_stats(self._h, C.byref(f), C.byref(p), C.byref(l)))
        return f.value, p.value, l.value

    def mfma_ceiling(self, iters: int = 20000, stream=0) -> float:
        """Achieved TFLOP/s of a register-only bf16 MFMA kernel on this device (measurement aid)."""
        out = C.c_double()
        self._check(self._l.sdstream_mfma_ceiling(self._h, iters, C.byref(out), stream or None))
        return out.value

    # ---- profiling
    def profile_enable(self, on: bool):
        self._check(self._l.sdstream_profile_enable(self._h, int(on)))

    def profile_reset(self):
        self._check(self._l.sdstream_profile_reset(self._h))

    def profile_read(self):
        buf = (ProfileEntry * 32)()
        n = self._check(self._l.sdstream_profile_read(self._h, buf, 32))
        return {buf[i].name.decode(): dict(launches=buf[i].launches, ms=buf[i].ms, flops=buf[i].flops,
                                           bytes=buf[i].bytes) for i in range(n)}
