"""Pins of the two compositions around the layer: per-channel difficulty migration between X
and W (the combination Sec. V names) and the GPT-2 MLP chain c_fc -> GELU -> c_proj (Sec. IV-C)."""
from fractions import Fraction as F

import numpy as np

import brute
from oracle import muxq_oracle as orc
from paper_2604_04701_amd import synth
from paper_2604_04701_amd.synth import Case


def test_smoothing_elements_against_exact_rationals():
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((6, 8)) * 9).astype(np.float16)
    W = (rng.standard_normal((8, 5)) * 0.05).astype(np.float16)
    f = rng.uniform(0.3, 7.0, size=8).astype(np.float32)
    Xs, Ws = orc.smooth(X, W, f)
    for m in range(6):
        for k in range(8):
            want = np.float16(float(brute.fl32(F(float(X[m, k])) / F(float(f[k])))))
            assert Xs[m, k] == want
    for k in range(8):
        for n in range(5):
            want = np.float16(float(brute.fl32(F(float(W[k, n])) * F(float(f[k])))))
            assert Ws[k, n] == want


def test_smoothing_by_powers_of_two_leaves_the_product_unchanged():
    X, W, _ = synth.make_case(Case("smooth_p2", 32, 64, 16, 4, (20.0, 60.0), 5))
    # factors 1..8: W f stays in fp16's normal range; entries of X that X / f would push into
    # the subnormal range (and so round) are cleared first
    f = np.exp2(np.random.default_rng(1).integers(0, 4, size=64)).astype(np.float32)
    X[np.abs(X) < np.float16(2.0 ** -10)] = 0
    Xs, Ws = orc.smooth(X, W, f)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    assert np.array_equal(Xs.astype(np.float64) @ Ws.astype(np.float64), exact)
    # general factors: each operand moves by at most half an fp16 unit in the last place
    f = np.random.default_rng(2).uniform(0.5, 4.0, size=64).astype(np.float32)
    Xs, Ws = orc.smooth(X, W, f)
    bound = (np.abs(X.astype(np.float64)) @ np.abs(W.astype(np.float64))) * (2 * 2.0 ** -11 + 2.0 ** -20)
    assert (np.abs(Xs.astype(np.float64) @ Ws.astype(np.float64) - exact) <= bound + 1e-12).all()


def test_smoothing_moves_difficulty_and_combines_with_the_decomposition():
    # activations with a few loud channels; factors f = sqrt(max|X_k| / max|W_k|)
    case = Case("smooth_mix", 256, 256, 96, 6, (20.0, 60.0), 11)
    X, W, planted = synth.make_case(case)
    cx = np.abs(X.astype(np.float32)).max(axis=0)
    cw = np.abs(W.astype(np.float32)).max(axis=1)
    f = np.sqrt(cx / cw).astype(np.float32)
    f = f / np.float32(np.median(f))                 # keep the quiet channels where they are
    Xs, Ws = orc.smooth(X, W, f)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    db = lambda o: orc.sqnr_db(o["y32"], exact)
    naive = db(orc.linear(X, W, r_cap=0))
    muxq = db(orc.linear(X, W))
    smooth_naive = db(orc.linear(Xs, Ws, r_cap=0))
    smooth_muxq = db(orc.linear(Xs, Ws, threshold=6.0))
    # the loud channels shrink in X' (difficulty moved to W'), so the naive quantiser gains
    assert np.abs(Xs[:, planted].astype(np.float32)).max() < np.abs(X[:, planted].astype(np.float32)).max() / 3
    assert smooth_naive > naive + 3.0
    # the decomposition still applies to whatever stays above the threshold after smoothing,
    # and never costs accuracy against the naive quantiser on the same operands
    assert smooth_muxq >= smooth_naive - 0.05 and muxq > naive + 3.0


def test_mlp_chain_is_the_composition_of_its_pinned_parts():
    rng = np.random.default_rng(9)
    X, W1, _ = synth.make_case(Case("mlp1", 24, 32, 64, 2, (20.0, 40.0), 21))
    W2 = synth.make_w(64, 32, rng)
    b1 = (0.1 * rng.standard_normal(64)).astype(np.float16)
    b2 = (0.1 * rng.standard_normal(32)).astype(np.float16)
    g, o2 = orc.mlp(X, W1, b1, W2, b2, w_gran="channel")
    y1 = orc.linear(X, W1, bias16=b1, w_gran="channel")["y16"]
    assert y1.dtype == np.float16
    g_want = orc.gelu_tanh(y1)
    assert np.array_equal(g, g_want)
    o2_want = orc.linear(g_want, W2, bias16=b2, w_gran="channel")
    assert np.array_equal(o2["y16"], o2_want["y16"]) and np.array_equal(o2["body_q"], o2_want["body_q"])
    # the hidden activation is what sets the second layer's outlier list: gelu(y) <= y for y > 0,
    # so no hidden channel can exceed the first layer's output maximum
    assert np.abs(g.astype(np.float32)).max() <= np.abs(y1.astype(np.float32)).max()
