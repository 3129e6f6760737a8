"""CPU-side checks of the C ABI: the built library exports every function the header declares, and the host half
of the similarity filter agrees with the oracle (no GPU call is made here)."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sdstream.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdstream_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2312_12491_amd import binding
    names = _declared()
    assert len(names) >= 20
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.exported_symbols()) == names      # the Python binding wraps all of them, and nothing else


def test_create_rejects_bad_arguments_without_a_gpu_call():
    from paper_2312_12491_amd import binding
    l = binding.lib()
    assert l.sdstream_create(None, None) == -1
    assert b"null" in l.sdstream_last_error(None)
    from workloads import CONFIGS
    cfg = binding.config_from_dict(dict(CONFIGS[1]["unet"], head_dim=0), (8, 8), "fp32", 2, 1, 0)   # no head field set
    h = ctypes.c_void_p()
    assert l.sdstream_create(ctypes.byref(cfg), ctypes.byref(h)) == -1 and not h.value
    cfg = binding.config_from_dict(CONFIGS[1]["unet"], (9, 8), "fp32", 2, 1, 0)                    # 9 not divisible by 2
    assert l.sdstream_create(ctypes.byref(cfg), ctypes.byref(h)) == -1 and not h.value
    assert l.sdstream_step(None, None, None, None, 0, None, 1.0, 1.0, None, None, None) == -1


def test_ssf_decide_matches_the_oracle():
    from oracle import ssf as F
    from paper_2312_12491_amd import ssf_decide
    rng = np.random.default_rng(0)
    for k in range(2000):
        a = rng.integers(0, 256, 300, dtype=np.uint8)
        b = np.clip(a.astype(np.int64) + rng.integers(-12, 13, 300), 0, 255).astype(np.uint8) if k % 3 else a
        d, nt, nr = F.sums(a, b)
        eta = [0.9, 0.98, 1.0][k % 3]
        skip, p = ssf_decide(d, nt, nr, eta, 7000, k)
        want_p = F.skip_probability(F.cosine(d, nt, nr), eta)
        assert p == want_p
        assert skip == (F.uniform(7000, k) < want_p)
    assert ssf_decide(0, 0, 5, 0.5, 1, 1) == (False, 0.0)
    assert ssf_decide(25, 25, 25, 0.98, 1, 1)[1] == 1.0
    assert ssf_decide(25, 25, 25, 1.0, 1, 1) == (False, 0.0)


def test_ssf_decide_hard_matches_the_oracle():
    # host half of the hard-threshold filter (no GPU needed): skip exactly when S_C > eta
    from oracle import ssf as F
    from paper_2312_12491_amd import ssf_decide_hard
    rng = np.random.default_rng(12)
    for k in range(300):
        a = rng.integers(0, 256, size=200, dtype=np.int64)
        b = np.clip(a + rng.integers(-30, 31, size=200), 0, 255)
        d, nt, nr = int((a * b).sum()), int((a * a).sum()), int((b * b).sum())
        eta = float(rng.uniform(0.9, 1.0))
        skip, sc = ssf_decide_hard(d, nt, nr, eta)
        want = F.cosine(d, nt, nr)
        assert sc == want or abs(sc - want) <= 2.3e-16 * want
        assert skip == (want > eta)
    assert ssf_decide_hard(0, 0, 5, 0.5) == (False, 0.0)
    assert ssf_decide_hard(25, 25, 25, 0.98) == (True, 1.0)
    assert ssf_decide_hard(25, 25, 25, 1.0) == (False, 1.0)


def test_multiply_high_division_is_exact():
    # the GEMM kernels divide block and pixel indices by launch-time constants with one multiply-high
    # (round-up method): same arithmetic as make_fastdiv / fast_div in csrc/common.h, checked against // here
    import random

    def make(d):
        l = 0 if d == 1 else (d - 1).bit_length()
        return ((((1 << l) - d) << 32) // d + 1, min(l, 1), max(l - 1, 0))

    def fdiv(x, f):
        m, sh1, sh2 = f
        t = (m * x) >> 32
        return ((t + (((x - t) & 0xFFFFFFFF) >> sh1)) & 0xFFFFFFFF) >> sh2

    rng = random.Random(7)
    for d in list(range(1, 700)) + [4095, 4096, 4097, 9216, 16384, 65537, 147456, (1 << 31) - 1]:
        f = make(d)
        assert f[0] < (1 << 32)
        xs = [0, 1, d - 1, d, d + 1, 2 * d - 1, (1 << 31) - 1, (1 << 31) - d] + [rng.randrange(1 << 31) for _ in range(50)]
        for x in xs:
            if 0 <= x < (1 << 31):
                assert fdiv(x, f) == x // d, (d, x)
