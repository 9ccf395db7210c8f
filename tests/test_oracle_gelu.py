"""Pins of the oracle's GELU (the producer of X in the MLP of Sec. IV-C's GPT-2 blocks)."""
import numpy as np
import torch

from oracle import muxq_oracle as orc


def all_finite_fp16():
    bits = np.arange(1 << 16, dtype=np.uint16)
    v = bits.view(np.float16)
    return v[np.isfinite(v)]


def test_matches_the_library_routine_on_every_fp16_value():
    y = all_finite_fp16()
    ref = torch.nn.functional.gelu(torch.from_numpy(y.astype(np.float64)), approximate="tanh")
    ref16 = ref.numpy().astype(np.float16)
    got = orc.gelu_tanh(y)
    assert got.dtype == np.float16
    assert (got.view(np.uint16) == ref16.view(np.uint16)).all()


def test_closed_forms_and_limits():
    assert orc.gelu_tanh(np.float16(0.0)) == 0.0
    big = np.array([6.0, 10.0, 100.0, 65504.0], dtype=np.float16)
    assert (orc.gelu_tanh(big) == big).all()                    # 1 + tanh -> 2 long before fp16 notices
    assert (np.abs(orc.gelu_tanh(-big).astype(np.float64)) < 1e-6).all()
    # tanh is odd: gelu(y) - gelu(-y) = y before the rounding to fp16
    y = np.linspace(-5.0, 5.0, 2001).astype(np.float16).astype(np.float64)
    u = np.sqrt(2.0 / np.pi) * (y + 0.044715 * y ** 3)
    g = lambda t, uu: 0.5 * t * (1.0 + np.tanh(uu))
    assert np.allclose(g(y, u) - g(-y, -u), y, rtol=0, atol=1e-15)
    # a dropped cubic term, a wrong constant or the erf form would move these (values to 6 digits)
    pts = np.array([-2.0, -1.0, -0.5, 0.5, 1.0, 2.0, 3.0], dtype=np.float16)
    want = np.array([-0.0454023, -0.158808, -0.154286, 0.345714, 0.841192, 1.95460, 2.99636])
    assert np.allclose(orc.gelu_tanh(pts).astype(np.float64), want, rtol=6e-4, atol=0)


def test_minimum_and_monotone_right_of_it():
    # the function has one minimum, near y = -0.752, of about -0.17004 (fp16 ties around it), and
    # rises from there on
    y = all_finite_fp16()
    y = np.sort(y[(y > -4) & (y < 4)])
    g = orc.gelu_tanh(y).astype(np.float64)
    k = int(np.argmin(g))
    assert abs(float(y[k]) + 0.752) < 0.03 and abs(g[k] + 0.17004) < 2e-4
    assert (np.diff(g[k:]) >= 0).all() and (np.diff(g[:k + 1]) <= 0).all()
