"""Properties the paper and the mathematics fix, checked on the CPU oracle.

Each test names the passage it comes from.  Independent re-computations use
numpy integer/float64 library routines or are written out here; none of them
calls the oracle function it is checking.
"""
import numpy as np
import pytest

from oracle import muxq_oracle as orc
from paper_2604_04701_amd import synth


def small_case(seed=11, M=96, K=160, N=72, r=5, gain=(20.0, 100.0)):
    c = synth.Case("t", M, K, N, r, gain, seed)
    X, W, ch = synth.make_case(c)
    return X, W, ch


def naive_int8_numpy(X16, W16, w_gran="tensor"):
    """Plain Eq. 1-3 written with numpy (np.rint rounds half to even)."""
    X = X16.astype(np.float32)
    W = W16.astype(np.float32)
    ax = np.float32(np.abs(X).max())
    sx = ax / np.float32(127)
    ix = np.float32(127) / ax if ax > 0 else np.float32(0)
    xq = np.clip(np.rint(X * ix), -127, 127).astype(np.int64)
    if w_gran == "tensor":
        aw = np.float32(np.abs(W).max()) * np.ones(W.shape[1], np.float32)
    else:
        aw = np.abs(W).max(axis=0).astype(np.float32)
    sw = aw / np.float32(127)
    iw = np.where(aw > 0, np.float32(127) / np.where(aw > 0, aw, 1), 0).astype(np.float32)
    wq = np.clip(np.rint(W * iw[None, :]), -127, 127).astype(np.int64)
    acc = xq @ wq
    y = (sx * sw)[None, :].astype(np.float32) * acc.astype(np.float32)
    return xq, wq, acc, y.astype(np.float32)


@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
@pytest.mark.parametrize("how", ["threshold_inf", "r_cap_0", "exp_0", "no_outliers_in_data"])
def test_zero_outliers_reduces_to_naive_int8(how, w_gran):
    # With no outlier channel MUXQ is exactly per-tensor abs-max INT8 (Eq. 1-3).
    X, W, _ = small_case()
    kw = dict(threshold=6.0, e=2, r_cap=64)
    if how == "threshold_inf":
        kw["threshold"] = float("inf")
    elif how == "r_cap_0":
        kw["r_cap"] = 0
    elif how == "exp_0":
        kw["e"] = 0
    else:
        X = np.clip(X, -6, 6).astype(np.float16)
    o = orc.linear(X, W, w_gran=w_gran, **kw)
    xq, wq, acc, y = naive_int8_numpy(X, W, w_gran)
    assert (o["body_q"] == xq).all()
    assert (o["w_q"] == wq).all()
    assert (o["acc"] == acc).all()
    assert (o["y32"] == y).all()
    if how != "exp_0":
        assert o["n_used"] == 0


@pytest.mark.parametrize("e", [1, 2, 3, 5])
def test_decomposition_reconstructs_x_exactly(e):
    # Eq. 6: X_outlier = Body_outlier + (2^e - 1) Aux, exact in fp32 for fp16 data.
    X, W, ch = small_case(seed=12)
    X[0, ch[0]] = np.float16(6e-8) * 3           # subnormal entry inside an outlier column
    o = orc.linear(X, threshold=6.0, e=e)
    r = o["n_used"]
    idx = o["outlier_idx"][:r]
    assert set(ch.tolist()) <= set(idx.tolist())
    rec = orc.reconstruct(o["body"], np.ascontiguousarray(o["aux"]), o["outlier_idx"], r, e)
    assert (rec == X.astype(np.float32)[:, idx]).all()
    # and independently of the oracle's own reconstruct step
    c = np.float32(2 ** e - 1)
    assert (o["body"][:, idx] + c * o["aux"] == X.astype(np.float32)[:, idx]).all()
    mask = np.ones(X.shape[1], bool)
    mask[idx] = False
    assert (o["body"][:, mask] == X.astype(np.float32)[:, mask]).all()
    assert (o["body"][:, idx] * np.float32(2 ** e) == X.astype(np.float32)[:, idx]).all()


@pytest.mark.parametrize("e", [1, 2, 3])
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_accumulators_match_integer_matmul(e, w_gran):
    # Eq. 7 in integers: acc = sum_k f_k body_q[m,k] w_q[k,n], f_k = 2^e on outlier columns.
    X, W, _ = small_case(seed=13, M=200, K=320, N=130, r=9)
    o = orc.linear(X, W, e=e, w_gran=w_gran)
    f = np.ones(X.shape[1], np.int64)
    f[o["outlier_idx"][:o["n_used"]]] = 2 ** e
    ref = (o["body_q"].astype(np.int64) * f[None, :]) @ o["w_q"].astype(np.int64)
    assert (o["acc"].astype(np.int64) == ref).all()
    assert (o["acc_body"].astype(np.int64)
            == o["body_q"].astype(np.int64) @ o["w_q"].astype(np.int64)).all()


def test_exp_factor_one_is_a_plain_sum_of_two_products():
    # Sec. III-C: with exp factor 1 the outputs of the two products are simply added.
    X, W, _ = small_case(seed=14)
    o = orc.linear(X, W, e=1)
    assert o["n_used"] > 0
    assert (o["acc"] == o["acc_body"] + o["acc_aux"]).all()


def test_code_invariants():
    X, W, _ = small_case(seed=15)
    o = orc.linear(X, W, w_gran="channel")
    r = o["n_used"]
    idx = o["outlier_idx"][:r]
    assert np.abs(o["body_q"]).max() == 127 and o["body_q"].min() >= -127
    assert (np.abs(o["w_q"]).max(axis=0) == 127).all() and o["w_q"].min() >= -127
    assert (o["aux_q"] == o["body_q"][:, idx]).all()          # Eq. 5 on codes
    # the Body abs-max can be read off the column maxima alone
    mult = np.ones(X.shape[1], np.float32)
    mult[idx] = 0.25
    assert np.float32((o["col_absmax"] * mult).max()) == o["amax_body"]


def test_quantiser_error_is_half_a_step():
    # abs-max quantiser closed form: |v - s q| <= s/2 (plus fp32 rounding slack), no clipping.
    X, W, _ = small_case(seed=16)
    o = orc.linear(X, W, w_gran="channel")
    s = float(o["s_x"][0])
    err = np.abs(o["body"].astype(np.float64) - s * o["body_q"].astype(np.float64))
    assert err.max() <= 0.5 * s * (1 + 1e-5)
    assert err.max() >= 0.4 * s                      # the bound is tight, not vacuous
    sw = o["s_w"].astype(np.float64)[None, :]
    errw = np.abs(W.astype(np.float64) - sw * o["w_q"].astype(np.float64))
    assert (errw <= 0.5 * sw * (1 + 1e-5)).all()


def test_end_to_end_error_bound_and_muxq_beats_naive():
    # |Y - XW| is bounded by the propagated half-step errors, and shrinking the outlier
    # columns by 2^e shrinks the activation step by min(2^e, amax_outlier/amax_normal)
    # (Sec. II-B, Fig. 3; Sec. III-B), so MUXQ's error is below naive INT8's.
    X, W, ch = small_case(seed=17, M=128, K=256, N=96, r=6, gain=(60.0, 60.0))
    exact = X.astype(np.float64) @ W.astype(np.float64)
    o = orc.linear(X, W)
    n = orc.linear(X, W, threshold=float("inf"))
    f = np.ones(X.shape[1])
    f[o["outlier_idx"][:o["n_used"]]] = 4.0
    sx, sw = float(o["s_x"][0]), float(o["s_w"][0])
    bound = ((0.5 * sx * f)[None, :] @ np.abs(W.astype(np.float64))
             + 0.5 * sw * (np.abs(o["body"].astype(np.float64)) * f[None, :]).sum(1, keepdims=True)
             + 0.25 * sx * sw * f.sum())
    err = np.abs(o["y32"].astype(np.float64) - exact)
    assert (err <= bound * (1 + 1e-4) + 1e-6).all()
    e_muxq = np.linalg.norm(o["y32"] - exact)
    e_naive = np.linalg.norm(n["y32"] - exact)
    assert e_muxq < e_naive
    step_ratio = float(n["s_x"][0]) / sx
    assert abs(step_ratio - 4.0) < 1e-6              # outliers (x60) >> 4 x normal max
    assert e_naive / e_muxq > 1.5
    # fp16 output stays within the tolerance the GPU parity tests use
    assert np.abs(o["y16"].astype(np.float64) - o["y32"]).max() <= 1e-3 * np.abs(o["y32"]).max()


def test_metamorphic_permutations_and_padding():
    X, W, _ = small_case(seed=18, M=64, K=96, N=40, r=4)
    o = orc.linear(X, W)
    rng = np.random.default_rng(0)
    pm = rng.permutation(X.shape[0])
    op = orc.linear(X[pm], W)
    assert (op["acc"] == o["acc"][pm]).all() and (op["y32"] == o["y32"][pm]).all()
    pk = rng.permutation(X.shape[1])
    ok = orc.linear(np.ascontiguousarray(X[:, pk]), np.ascontiguousarray(W[pk]))
    assert (ok["acc"] == o["acc"]).all()
    Xz = np.concatenate([X, np.zeros((7, X.shape[1]), np.float16)])
    oz = orc.linear(Xz, W)
    assert (oz["acc"][:64] == o["acc"]).all() and (oz["acc"][64:] == 0).all()


def test_row_subset_matches_full_run():
    X, W, _ = small_case(seed=19)
    o = orc.linear(X, W, w_gran="channel")
    rows = [0, 5, 95, 17]
    s = orc.linear(X, W, w_gran="channel", rows=rows)
    assert (s["acc"] == o["acc"][rows]).all() and (s["y32"] == o["y32"][rows]).all()


def test_config1_planted_channels_are_found():
    case = synth.config_cases(1)[0]
    X, W, ch = synth.make_case(case)
    o = orc.linear(X, W)
    assert o["outlier_idx"][:o["n_used"]].tolist() == ch.tolist()
    assert o["n_used"] == 6


def test_synth_is_deterministic():
    case = synth.config_cases(2)[1]
    X1, W1, c1 = synth.make_case(case)
    X2, W2, c2 = synth.make_case(case)
    assert (X1 == X2).all() and (W1 == W2).all() and (c1 == c2).all()
    assert X1.dtype == np.float16 and X1.shape == (1024, 768) and W1.shape == (768, 768)


# ---- per-token activation scales and narrower codes (Sec. II-A per-vector setting; Tables 1-2) ----

def _varied_rows_case(seed=77, M=48, K=96, N=40, r=4):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)) * rng.uniform(0.05, 4.0, (M, 1))   # tokens of very different size
    ch = np.sort(rng.choice(K, r, replace=False))
    X[:, ch] *= rng.uniform(20, 100, r)
    W = rng.standard_normal((K, N)) * 0.02
    return X.astype(np.float16), W.astype(np.float16), ch


def test_per_token_equals_per_tensor_when_rows_share_their_absmax():
    X, W, ch = _varied_rows_case()
    X = X.copy()
    X[:, ch[0]] = np.float16(32768.0)         # every row's Body abs-max sits on this outlier channel
    a = orc.linear(X, W, x_gran="tensor")
    b = orc.linear(X, W, x_gran="token")
    assert (b["s_x"] == a["s_x"][0]).all()
    for k in ("body_q", "aux_q", "acc", "y16"):
        assert (a[k] == b[k]).all(), k


def test_per_token_rows_depend_only_on_their_own_row_and_the_outlier_set():
    X, W, ch = _varied_rows_case(seed=78)
    full = orc.linear(X, W, x_gran="token")
    keep = [0, 5, 6, 17, 40]
    # the kept rows plus one row carrying every channel's abs-max, so that the same
    # channels are detected; only the kept rows are compared
    Xs = np.concatenate([X[keep], np.abs(X).max(axis=0, keepdims=True)])
    sub = orc.linear(Xs, W, x_gran="token")
    assert sub["outlier_idx"].tolist() == full["outlier_idx"].tolist()
    assert (sub["body_q"][:-1] == full["body_q"][keep]).all()
    assert (sub["s_x"][:-1] == full["s_x"][keep]).all()
    assert (sub["acc"][:-1] == full["acc"][keep]).all()
    assert (sub["y16"][:-1] == full["y16"][keep]).all()


def test_per_token_half_step_bound_and_full_range_per_row():
    X, W, _ = _varied_rows_case(seed=79)
    o = orc.linear(X, W, x_gran="token")
    body, s = o["body"].astype(np.float64), o["s_x"].astype(np.float64)[:, None]
    assert (np.abs(o["body_q"]).max(axis=1) == 127).all()
    assert (np.abs(body - s * o["body_q"]) <= s / 2 * (1 + 2.0 ** -21)).all()


def test_per_token_is_more_accurate_when_token_sizes_vary():
    # the per-vector rows of Table 1 sit below the per-tensor rows; same ordering here
    X, W, _ = _varied_rows_case(seed=80, M=64, K=128, N=48)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    err = {}
    for xg in ("tensor", "token"):
        o = orc.linear(X, W, x_gran=xg, w_gran="channel")
        err[xg] = np.linalg.norm(o["y32"].astype(np.float64) - exact)
    assert err["token"] < 0.6 * err["tensor"]


@pytest.mark.parametrize("bits", [7, 6, 5])
def test_fewer_activation_bits_double_the_step_and_muxq_keeps_its_lead(bits):
    # Table 1, IA 7/6/5: the quantisation step of Body doubles per bit removed, and the
    # decomposition keeps shrinking it by 2^exp where the outliers set the range
    cfg = synth.Case("bits", 96, 256, 64, 6, (60.0, 60.0), 81)
    X, W, _ = synth.make_case(cfg)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    m8 = orc.linear(X, W, ia_bits=8)
    mb = orc.linear(X, W, ia_bits=bits)
    nb = orc.linear(X, W, ia_bits=bits, threshold=float("inf"))
    q8, qb = 127.0, float(2 ** (bits - 1) - 1)
    assert abs(float(mb["s_x"][0]) / float(m8["s_x"][0]) - q8 / qb) < 1e-6
    assert abs(float(nb["s_x"][0]) / float(mb["s_x"][0]) - 4.0) < 1e-6      # 2^exp, exp = 2
    e_m = np.linalg.norm(mb["y32"].astype(np.float64) - exact)
    e_n = np.linalg.norm(nb["y32"].astype(np.float64) - exact)
    # the lead shrinks as the step grows past the normal channels' own size (at 5 bits both
    # variants round most of them to zero), as the IA5 column of Table 1 shows, but it stays
    assert e_m < (0.6 if bits >= 7 else 0.95) * e_n
    assert np.abs(mb["body_q"]).max() == qb and np.abs(mb["aux_q"]).max() <= qb


@pytest.mark.parametrize("w_bits", [5, 4])
def test_fewer_weight_bits(w_bits):
    # Table 2: W 5 / 4 bits; codes fill the narrower symmetric range, per tensor and per channel
    cfg = synth.Case("wbits", 32, 128, 72, 3, (50.0, 50.0), 82)
    X, W, _ = synth.make_case(cfg)
    qw = 2 ** (w_bits - 1) - 1
    for gran in ("tensor", "channel"):
        p8 = orc.quantize_weight(W, gran, 8)
        pb = orc.quantize_weight(W, gran, w_bits)
        assert np.abs(pb["w_q"]).max() == qw
        if gran == "channel":
            assert (np.abs(pb["w_q"]).max(axis=0) == qw).all()
        ratio = pb["s_w"].astype(np.float64) / p8["s_w"].astype(np.float64)
        assert np.allclose(ratio, 127.0 / qw, rtol=1e-6)
        W64 = W.astype(np.float64)
        assert (np.abs(W64 - pb["s_w"].astype(np.float64) * pb["w_q"]) <=
                pb["s_w"].astype(np.float64) / 2 * (1 + 2.0 ** -21)).all()
