"""Pins of the CPU oracle against exact brute force and the worked example.

The brute force (tests/brute.py) is written in Python rationals/ints with its
own binary32 rounding; it shares nothing with the C oracle.  Cases are tiny
and adversarial: rounding ties, threshold edge, capacity truncation, zero
tensors, zero weight columns, every exp factor, both weight granularities.
"""
import json
import os
import struct
from fractions import Fraction as F

import numpy as np
import pytest

import brute
from oracle import muxq_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "w1_worked_example.json")


def to_frac(a16):
    return [[F(float(v)) for v in row] for row in np.asarray(a16, np.float16)]


def check_against_brute(X16, W16, *, T=6.0, e=2, r_cap=64, w_gran="tensor", bias16=None,
                        x_gran="tensor", ia_bits=8, w_bits=8, static_idx=None):
    o = orc.linear(X16, W16, threshold=T, e=e, r_cap=r_cap, w_gran=w_gran, bias16=bias16,
                   x_gran=x_gran, ia_bits=ia_bits, w_bits=w_bits, static_idx=static_idx)
    b = brute.muxq_linear(to_frac(X16), to_frac(W16), T=F(T), e=e, r_cap=r_cap,
                          w_gran="tensor" if w_gran == "tensor" else "channel",
                          bias=None if bias16 is None else [F(float(v)) for v in bias16],
                          qx=2 ** (ia_bits - 1) - 1, qw=2 ** (w_bits - 1) - 1, x_gran=x_gran,
                          idx_given=static_idx)
    r = len(b["idx"])
    assert o["n_used"] == r and o["n_total"] == b["n_total"]
    assert o["outlier_idx"][:r].tolist() == b["idx"]
    assert (o["outlier_idx"][r:] == -1).all()
    assert [F(float(v)) for v in o["col_absmax"]] == b["colmax"]
    assert [[F(float(v)) for v in row] for row in o["body"]] == b["body"]
    if x_gran == "tensor":
        assert F(float(o["s_x"][0])) == b["s_x"]
        assert F(float(o["inv_x"][0])) == b["inv_x"]
    else:
        assert [F(float(v)) for v in o["s_x"]] == b["s_x"]
        assert [F(float(v)) for v in o["inv_x"]] == b["inv_x"]
    assert o["body_q"].tolist() == b["body_q"]
    assert o["aux_q"].reshape(len(b["aux_q"]), r).tolist() == [row[:r] for row in b["aux_q"]]
    assert o["w_q"].tolist() == b["w_q"]
    sw = o["s_w"] if o["s_w"].size > 1 else np.repeat(o["s_w"], len(b["s_w"]))
    assert [F(float(v)) for v in sw] == b["s_w"]
    assert o["acc"].tolist() == b["acc"]
    assert [[F(float(v)) for v in row] for row in o["y32"]] == b["y32"]
    return o, b


def test_fl32_helper_matches_binary32_encoding():
    # the brute force's own rounding against the platform's binary32 encoding
    rng = np.random.default_rng(1)
    for _ in range(2000):
        num = int(rng.integers(-10**12, 10**12))
        den = int(rng.integers(1, 10**9))
        fr = F(num, den)
        via_struct = struct.unpack("f", struct.pack("f", num / den))[0]
        # num/den is already rounded to binary64; only compare when that step is exact enough
        got = float(brute.fl32(fr))
        assert got == via_struct or abs(got - via_struct) <= abs(via_struct) * 2**-23
    assert brute.fl32(F(1, 3)) == F(11184811, 2**25)
    assert brute.fl32(F(2**24 + 1)) == F(2**24)          # tie -> even
    assert brute.fl32(F(2**24 + 3)) == F(2**24 + 4)      # tie -> even (up)
    assert brute.fl32(F(1, 2**149)) == F(1, 2**149)      # smallest subnormal
    assert brute.rne(F(5, 2)) == 2 and brute.rne(F(7, 2)) == 4 and brute.rne(F(-5, 2)) == -2


def test_worked_example_golden():
    g = json.load(open(GOLD))
    X = np.array(g["X"], np.float16)
    W = np.array(g["W"], np.float16)
    o = orc.linear(X, W, threshold=g["threshold"], e=g["exp"])
    assert o["col_absmax"].tolist() == g["col_absmax"]
    assert o["outlier_idx"][:o["n_used"]].tolist() == g["outlier_idx"]
    assert o["body"].tolist() == g["body"]
    assert float(o["amax_body"]) == g["amax_body"] and float(o["inv_x"][0]) == g["inv_x"]
    assert o["body_q"].tolist() == g["body_q"]
    assert o["aux_q"].tolist() == g["aux_q"]
    assert o["w_q"].tolist() == g["w_q"]
    assert o["acc_body"].tolist() == g["acc_body"]
    assert o["acc_aux"].tolist() == g["acc_aux"]
    assert o["acc"].tolist() == g["acc"]
    assert o["y16"].astype(np.float64).tolist() == g["y16"]
    # plain Eq. 1-3 (no outlier handling) on the same data
    naive = orc.linear(X, W, threshold=float("inf"), e=g["exp"])
    assert naive["body_q"].tolist() == g["naive_x_q"]
    assert naive["acc"].tolist() == g["naive_acc"]
    # the same example through the exact brute force
    check_against_brute(X, W, T=g["threshold"], e=g["exp"])


def test_rounding_ties_go_to_even():
    # abs-max 127/32 makes inv exactly 32: 0.078125*32 = 2.5 -> 2, 0.109375*32 = 3.5 -> 4
    X = np.array([[3.96875, 0.078125, 0.109375, -0.078125, -0.109375, 0.046875]], np.float16)
    W = np.eye(6, dtype=np.float16)
    o, _ = check_against_brute(X, W)
    assert float(o["inv_x"][0]) == 32.0
    assert o["body_q"].tolist() == [[127, 2, 4, -2, -4, 2]]   # 1.5 -> 2


def test_threshold_is_strict_and_on_raw_input():
    # exactly 6.0 is not an outlier; 6.0039 (next fp16) is
    X = np.array([[6.0, 6.00390625, 1.0, -6.0], [0.5, -1.0, 2.0, -6.00390625]], np.float16)
    W = np.array([[1, 2], [3, -1], [0.5, 0.25], [-2, 1]], np.float16)
    o, _ = check_against_brute(X, W)
    assert o["outlier_idx"][:o["n_used"]].tolist() == [1, 3]


def test_capacity_truncation_keeps_lowest_indices():
    rng = np.random.default_rng(7)
    X = rng.standard_normal((5, 10)).astype(np.float16)
    X[:, [1, 4, 6, 9]] *= np.float16(40)
    W = (rng.standard_normal((10, 4)) * 0.1).astype(np.float16)
    o, _ = check_against_brute(X, W, r_cap=2)
    assert o["n_used"] == 2 and o["n_total"] == 4
    assert o["outlier_idx"].tolist() == [1, 4]
    check_against_brute(X, W, r_cap=0)


@pytest.mark.parametrize("e", [0, 1, 2, 3])
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_random_tiny_cases(e, w_gran):
    rng = np.random.default_rng(100 + e)
    for trial in range(6):
        M, K, N = int(rng.integers(1, 7)), int(rng.integers(1, 13)), int(rng.integers(1, 6))
        X = rng.standard_normal((M, K)).astype(np.float16)
        r = int(rng.integers(0, min(K, 4) + 1))
        if r:
            ch = rng.choice(K, r, replace=False)
            X[:, ch] *= rng.uniform(10, 100, r).astype(np.float16)
        W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
        bias = rng.standard_normal(N).astype(np.float16) if trial % 2 else None
        check_against_brute(X, W, e=e, w_gran=w_gran, bias16=bias)


def test_zero_activation_and_zero_weight_column():
    X = np.zeros((3, 4), np.float16)
    W = np.array([[1, 0], [2, 0], [3, 0], [-1, 0]], np.float16)
    o, _ = check_against_brute(X, W, w_gran="channel")
    assert (o["body_q"] == 0).all() and (o["y32"] == 0).all() and float(o["s_x"][0]) == 0.0
    assert float(o["s_w"][1]) == 0.0 and np.isfinite(o["y32"]).all()
    X = np.array([[1, -9, 2, 0.25]], np.float16)
    o, _ = check_against_brute(X, W, w_gran="channel", bias16=np.array([0.5, -1.5], np.float16))
    assert o["y32"][0, 1] == -1.5


def test_subnormal_and_extreme_fp16_inputs():
    tiny = np.float16(6e-8)          # smallest fp16 subnormal
    X = np.array([[tiny, -tiny, 0], [0, tiny, tiny]], np.float16)
    W = np.array([[1, -1], [0.5, 2], [4, 1]], np.float16)
    check_against_brute(X, W)
    X = np.array([[65504, -65504, 1.0, 3.0], [2.0, 60000, -1.0, 0.5]], np.float16)
    check_against_brute(X, np.array([[1, -1], [0.5, 2], [4, 1], [1, 1]], np.float16))


# ---- per-token activation scales (the per-vector setting of Sec. II-A, Fig. 2(a)) and
# ---- narrower code widths (the IA / W columns of Tables 1-2) ----

@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
@pytest.mark.parametrize("e", [0, 2, 3])
def test_per_token_random_tiny_cases(e, w_gran):
    rng = np.random.default_rng(300 + e)
    for trial in range(6):
        M, K, N = int(rng.integers(1, 7)), int(rng.integers(1, 13)), int(rng.integers(1, 6))
        X = (rng.standard_normal((M, K)) * rng.uniform(0.1, 3, (M, 1))).astype(np.float16)
        r = int(rng.integers(0, min(K, 4) + 1))
        if r:
            ch = rng.choice(K, r, replace=False)
            X[:, ch] *= rng.uniform(10, 100, r).astype(np.float16)
        if trial == 3:
            X[0] = 0                                     # an all-zero token: scale 0, codes 0
        W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
        bias = rng.standard_normal(N).astype(np.float16) if trial % 2 else None
        o, _ = check_against_brute(X, W, e=e, w_gran=w_gran, bias16=bias, x_gran="token")
        assert o["s_x"].shape == (M,)


def test_per_token_ties_and_capacity():
    # row 0: abs-max 127/32 -> inv exactly 32, ties 2.5 -> 2 and 3.5 -> 4; row 1 has its own scale
    X = np.array([[3.96875, 0.078125, 0.109375, -0.078125],
                  [1.984375, 0.0390625, 0.0546875, 0.5]], np.float16)
    o, _ = check_against_brute(X, np.eye(4, dtype=np.float16), x_gran="token")
    assert o["inv_x"].tolist() == [32.0, 64.0]
    assert o["body_q"].tolist() == [[127, 2, 4, -2], [127, 2, 4, 32]]
    rng = np.random.default_rng(8)
    X = rng.standard_normal((5, 10)).astype(np.float16)
    X[:, [1, 4, 6, 9]] *= np.float16(40)
    W = (rng.standard_normal((10, 4)) * 0.1).astype(np.float16)
    o, _ = check_against_brute(X, W, r_cap=2, x_gran="token")
    assert o["outlier_idx"].tolist() == [1, 4]


@pytest.mark.parametrize("ia_bits,w_bits", [(7, 8), (6, 8), (5, 8), (8, 5), (8, 4), (5, 4), (2, 2)])
@pytest.mark.parametrize("x_gran", ["tensor", "token"])
def test_bit_widths_random_tiny_cases(ia_bits, w_bits, x_gran):
    rng = np.random.default_rng(400 + 10 * ia_bits + w_bits)
    for trial in range(4):
        M, K, N = int(rng.integers(1, 6)), int(rng.integers(1, 11)), int(rng.integers(1, 5))
        X = rng.standard_normal((M, K)).astype(np.float16)
        if K > 2:
            X[:, int(rng.integers(0, K))] *= np.float16(50)
        W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
        o, _ = check_against_brute(X, W, w_gran="channel" if trial % 2 else "tensor",
                                   x_gran=x_gran, ia_bits=ia_bits, w_bits=w_bits)
        qx, qw = 2 ** (ia_bits - 1) - 1, 2 ** (w_bits - 1) - 1
        assert np.abs(o["body_q"]).max() <= qx and np.abs(o["w_q"]).max() <= qw
        assert np.abs(o["body_q"]).max() == qx and np.abs(o["w_q"]).max() == qw


@pytest.mark.parametrize("x_gran", ["tensor", "token"])
def test_static_outlier_lists(x_gran):
    # a list fixed offline: channels below the threshold in it are still decomposed,
    # channels above the threshold outside it are not, and the capacity rule applies
    rng = np.random.default_rng(77)
    for trial in range(6):
        M, K, N = int(rng.integers(1, 6)), int(rng.integers(3, 11)), int(rng.integers(1, 5))
        X = rng.standard_normal((M, K)).astype(np.float16)
        X[:, int(rng.integers(0, K))] *= np.float16(40)
        W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
        lst = sorted(rng.choice(K, size=int(rng.integers(0, K)), replace=False).tolist())
        o, b = check_against_brute(X, W, e=1 + trial % 3, w_gran="channel" if trial % 2 else "tensor",
                                   x_gran=x_gran, static_idx=lst, r_cap=64 if trial < 4 else 2)
        assert o["n_total"] == len(lst)
    # the list the magnitude test would have found gives the dynamic result ...
    X = rng.standard_normal((4, 9)).astype(np.float16)
    X[:, [2, 7]] *= np.float16(30)
    W = (rng.standard_normal((9, 3)) * 0.05).astype(np.float16)
    dyn = orc.linear(X, W, x_gran=x_gran)
    sta = orc.linear(X, W, x_gran=x_gran, static_idx=[2, 7])
    for key in ("outlier_idx", "body_q", "aux_q", "s_x", "acc", "y16"):
        assert (dyn[key] == sta[key]).all(), key
    # ... and the empty list is the naive quantiser
    naive = orc.linear(X, W, x_gran=x_gran, r_cap=0)
    empty = orc.linear(X, W, x_gran=x_gran, static_idx=[])
    assert empty["n_used"] == 0 and (naive["body_q"] == empty["body_q"]).all()
    assert (naive["y16"] == empty["y16"]).all()
