"""Pins of the oracle's second route (Sec. IV-C: quantise, dequantise, multiply in floating
point) and of the accuracy figure built on it.  The integer route (Eq. 7 on codes, Eq. 3)
and this route share only the quantiser; their agreement checks the gather of the Aux
weights, the (2^e - 1) recombination and the dequantisation against plain fp64 algebra."""
import numpy as np
import pytest

from oracle import muxq_oracle as orc
from paper_2604_04701_amd import synth

CASE = synth.Case("eval", 192, 320, 136, 5, (20.0, 100.0), 11)
SETTINGS = [("tensor", "tensor", 8, 8), ("tensor", "channel", 8, 8), ("token", "channel", 8, 8),
            ("tensor", "tensor", 6, 8), ("token", "channel", 5, 8), ("tensor", "tensor", 8, 4),
            ("token", "tensor", 7, 5)]


@pytest.mark.parametrize("x_gran,w_gran,ia_bits,w_bits", SETTINGS)
@pytest.mark.parametrize("e", [1, 2, 3])
def test_float_route_equals_integer_route(x_gran, w_gran, ia_bits, w_bits, e):
    X, W, _ = synth.make_case(CASE)
    o = orc.linear(X, W, e=e, x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits, w_bits=w_bits)
    y = orc.fake_quant_linear(X, W, e=e, x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits, w_bits=w_bits)
    assert o["n_used"] == CASE.r
    # Eq. 3 rounds the scale product and the result to binary32: two roundings, 2^-23 each
    assert np.abs(y - o["y32"]).max() <= 3 * 2.0 ** -23 * np.abs(y).max()
    # ... and the naive setting is the same statement without Aux
    o0 = orc.linear(X, W, r_cap=0, x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits, w_bits=w_bits)
    y0 = orc.fake_quant_linear(X, W, muxq=False, x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits,
                               w_bits=w_bits)
    assert np.abs(y0 - o0["y32"]).max() <= 3 * 2.0 ** -23 * np.abs(y0).max()


def test_float_route_dropping_the_aux_term_is_caught():
    # the pin above has teeth: without Eq. 6's Aux term the two routes are far apart
    X, W, _ = synth.make_case(CASE)
    o = orc.linear(X, W)
    s_x = float(o["s_x"][0])
    wp = orc.quantize_weight(W)
    y_no_aux = (s_x * o["body_q"].astype(np.float64)) @ (wp["w_q"].astype(np.float64) * float(wp["s_w"][0]))
    assert np.abs(y_no_aux - o["y32"]).max() > 0.1 * np.abs(o["y32"]).max()


def test_sqnr_closed_forms():
    rng = np.random.default_rng(0)
    y = rng.standard_normal((50, 40))
    assert orc.sqnr_db(y, y) == float("inf")
    assert abs(orc.sqnr_db(y * 1.01, y) - 40.0) < 1e-9          # relative error 1e-2 everywhere
    assert abs(orc.sqnr_db(np.zeros_like(y), y)) < 1e-12        # all signal lost: 0 dB
    assert abs(orc.sqnr_db(-y, y) + 20 * np.log10(2.0)) < 1e-9  # error twice the signal


@pytest.mark.parametrize("x_gran,w_gran", [("tensor", "tensor"), ("token", "channel")])
def test_decomposition_lowers_the_error_at_every_width(x_gran, w_gran):
    # the ordering Tables 1-2 report (MUXQ below naive at every IA / W width), on the
    # synthetic outlier-bearing activations that stand in for the GPT-2 ones
    X, W, _ = synth.make_case(synth.Case("acc", 256, 768, 512, 6, (20.0, 100.0), 3))
    ref = X.astype(np.float64) @ W.astype(np.float64)
    gaps = {}
    for ia_bits, w_bits in [(8, 8), (7, 8), (6, 8), (5, 8), (8, 5), (8, 4)]:
        kw = dict(x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits, w_bits=w_bits)
        m = orc.sqnr_db(orc.fake_quant_linear(X, W, muxq=True, **kw), ref)
        n = orc.sqnr_db(orc.fake_quant_linear(X, W, muxq=False, **kw), ref)
        assert m > n, (ia_bits, w_bits, m, n)
        gaps[(ia_bits, w_bits)] = m - n
    # shrinking the outliers by 2^2 buys about two bits of activation resolution at IA = 8
    assert gaps[(8, 8)] > 6.0
    # without outlier channels there is nothing to decompose: the two coincide exactly
    X0, W0, _ = synth.make_case(synth.Case("acc0", 64, 128, 72, 0, (1.0, 1.0), 4))
    a = orc.fake_quant_linear(X0, W0, muxq=True, x_gran=x_gran, w_gran=w_gran)
    b = orc.fake_quant_linear(X0, W0, muxq=False, x_gran=x_gran, w_gran=w_gran)
    assert (a == b).all()
