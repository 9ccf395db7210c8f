"""Helpers shared by the GPU parity tests: run the HIP library on one seeded
case and compare every stage with the CPU oracle."""
import numpy as np
import torch

from oracle import muxq_oracle as orc
from paper_2604_04701_amd import binding as B
from paper_2604_04701_amd import synth

Y_REL_TOL = 1e-2      # max |Y_gpu - Y_oracle| <= 1e-2 * max |Y_fp32|  (fp16 output)


def say(msg):
    print(msg, flush=True)


def run_gpu(X, W, *, w_gran="tensor", bias=None, threshold=6.0, e=2, r_cap=64, naive=False,
            want_acc=True, x_gran="tensor", ia_bits=8, w_bits=8, finite=True, aux_scale="shared"):
    dev = "cuda"
    Xd = torch.from_numpy(X).to(dev)
    Wd = torch.from_numpy(W).to(dev)
    M, K = X.shape
    N = W.shape[1]
    w_q, w_scale = B.muxq_quantize_weight(Wd, w_gran, bits=w_bits)
    rc = 0 if naive else r_cap
    ws = B.alloc_workspace(M, K, N, rc)
    ws.fill_(0xCD)                         # stale bytes must not leak into results
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev) if want_acc else None
    bd = torch.from_numpy(bias).to(dev) if bias is not None else None
    if naive:
        Y = B.muxq_linear_naive_int8(Xd, w_q, w_scale, N, w_gran, bias=bd, workspace=ws, dbg_acc=acc)
    else:
        Y = B.muxq_linear(Xd, w_q, w_scale, N, w_gran, bias=bd, threshold=threshold, exp=e,
                          r_cap=r_cap, workspace=ws, dbg_acc=acc, x_gran=x_gran, ia_bits=ia_bits,
                          aux_scale=aux_scale)
    torch.cuda.synchronize()
    lay = B.workspace_layout(M, K, N, rc)
    get = lambda name: B.ws_view(ws, lay, name, M, N, rc).cpu().numpy()
    body_raw = get("body_q")
    # The unlisted channels are stored as code + z (zero point of the call, or of the row):
    # check what comes with that, and take it off before comparing with the oracle's codes.
    unlisted = get("col_slot")[:K] < 0
    zrow = (np.full(M, int(get("zero_point")[0]), np.int32) if x_gran == "tensor"
            else get("zero_point_token").astype(np.int32))
    z = zrow if x_gran == "token" else int(zrow[0])
    assert (zrow >= 0).all() and (zrow <= 64).all() and (zrow % 2 == 0).all()
    if unlisted.any() and finite:
        sub = body_raw[:, :K][:, unlisted] if M * K < (1 << 28) else None
        if sub is not None:
            unb = sub.astype(np.int32) - zrow[:, None]
            cmax = np.abs(unb).max(axis=1) if x_gran == "token" else np.full(M, np.abs(unb).max())
            assert (zrow == np.minimum(cmax + (cmax & 1), (127 - cmax) & ~1)).all(), "zero point rule"
            assert sub.min() >= -127
            assert (sub.min(axis=1)[cmax <= 63] >= 0).all(), "non-negative codes"
    zmat_cols = np.where(unlisted, 1, 0).astype(np.int8)
    if x_gran == "tensor":
        body_raw[:, :K] -= (zmat_cols * np.int8(zrow[0]))
    else:
        body_raw[:, :K] -= zrow.astype(np.int8)[:, None] * zmat_cols[None, :]
    wq_full = B.unpack(w_q, N, lay.k_pad).cpu().numpy().astype(np.int64)
    row_sums = B.wq_row_sums(w_q, K, N).cpu().numpy()
    assert (row_sums == wq_full.sum(axis=1)).all(), "weight code sums"
    # with a per-call zero point cn carries a fixed offset of 2^14: the accumulators then start
    # at z * 2^14 and stay on one side of zero, and the epilogue's acc - z * cn removes it
    cn_offset = (1 << 14) if x_gran == "tensor" else 0
    assert (get("cn") == wq_full[:, :K][:, unlisted].sum(axis=1) + cn_offset).all(), "cn"
    out = dict(Y=Y.cpu().numpy(), w_q=B.unpack(w_q, N, lay.k_pad).cpu().numpy(), zero_point=z,
               w_scale=w_scale.cpu().numpy(),
               col_absmax=get("col_absmax"), outlier_idx=get("outlier_idx"),
               n_outliers=get("n_outliers"),
               x_scale=get("x_scale_token" if x_gran == "token" else "x_scale"), body_q=body_raw,
               aux_q=get("aux_q") if rc else None, w_aux=get("w_aux") if rc else None,
               acc=acc.cpu().numpy() if want_acc else None, k_pad=lay.k_pad,
               aux_scale=(get("aux_scale_token" if x_gran == "token" else "aux_scale")
                          if aux_scale == "own" else None))
    return out


def compare(g, o, K, N, r_cap, rows=None, what=""):
    """g: run_gpu output, o: oracle.linear output (possibly on a row subset)."""
    kp = g["k_pad"]
    r = o["n_used"]
    assert (g["col_absmax"][:K] == o["col_absmax"]).all(), f"{what}: col_absmax"
    assert g["n_outliers"].tolist() == [r, o["n_total"]], f"{what}: n_outliers"
    if r_cap:
        assert (g["outlier_idx"][:r_cap] == o["outlier_idx"]).all(), f"{what}: outlier_idx"
    if g["x_scale"].ndim == 2:            # per token: s_x[M] then the reciprocal forms
        assert (g["x_scale"][0] == o["s_x"]).all() and (g["x_scale"][1] == o["inv_x"]).all(), \
            f"{what}: per-token x_scale"
    else:
        assert g["x_scale"][0] == o["s_x"][0] and g["x_scale"][1] == o["inv_x"][0], f"{what}: x_scale"
    assert (g["body_q"][:, :K] == o["body_q"]).all(), f"{what}: body_q"
    assert (g["body_q"][:, K:] == 0).all(), f"{what}: body_q K padding"
    if r_cap:
        assert (g["aux_q"][:, :r] == o["aux_q"]).all(), f"{what}: aux_q"
        assert (g["aux_q"][:, r:] == 0).all(), f"{what}: aux_q padding"
        idx = o["outlier_idx"][:r]
        assert (g["w_aux"][:, :r] == o["w_q"][idx, :].T).all(), f"{what}: w_aux"
        assert (g["w_aux"][:, r:] == 0).all(), f"{what}: w_aux padding"
    assert (g["w_q"][:, :K] == o["w_q"].T).all(), f"{what}: w_q"
    assert (g["w_q"][:, K:] == 0).all(), f"{what}: w_q K padding"
    assert (g["w_scale"] == o["s_w"]).all(), f"{what}: w_scale"
    sel = slice(None) if rows is None else np.asarray(rows)
    assert (g["acc"][sel] == o["acc"]).all(), f"{what}: INT32 accumulators"
    yg = g["Y"][sel].astype(np.float32)
    tol = Y_REL_TOL * float(np.abs(o["y32"]).max())
    err = float(np.abs(yg - o["y32"]).max()) if o["y32"].size else 0.0
    assert err <= tol, f"{what}: Y max abs err {err} > {tol}"
    # same op order on both sides: the fp16 results are expected to agree exactly
    same = (g["Y"][sel] == o["y16"]) | (np.isnan(g["Y"][sel]) & np.isnan(o["y16"]))
    assert same.all(), f"{what}: Y not bit-identical to the oracle ({(~same).sum()} elements)"


def check_case(case: synth.Case, rows=None, bias_seed=None, **over):
    X, W, _ = synth.make_case(case)
    kw = dict(w_gran=case.w_gran, threshold=case.threshold, e=case.exp, r_cap=case.r_cap)
    kw.update(over)
    bias = None
    if bias_seed is not None:
        bias = np.random.default_rng(bias_seed).standard_normal(case.N).astype(np.float16)
    say(f"[case] {case.name} M={case.M} K={case.K} N={case.N} r={case.r} seed={case.seed} {kw}")
    g = run_gpu(X, W, bias=bias, **kw)
    o = orc.linear(X, W, threshold=kw["threshold"], e=kw["e"], r_cap=kw["r_cap"],
                   w_gran=kw["w_gran"], bias16=bias, rows=rows, x_gran=kw.get("x_gran", "tensor"),
                   ia_bits=kw.get("ia_bits", 8), w_bits=kw.get("w_bits", 8))
    compare(g, o, case.K, case.N, kw["r_cap"], rows=rows, what=case.name)
    return g, o


def check_plain_y(case: synth.Case, rows=None, bias_seed=None, **over):
    """muxq_linear as a user calls it (no accumulator export): Y against the oracle."""
    X, W, _ = synth.make_case(case)
    kw = dict(w_gran=case.w_gran, threshold=case.threshold, e=case.exp, r_cap=case.r_cap)
    kw.update(over)
    bias = None
    if bias_seed is not None:
        bias = np.random.default_rng(bias_seed).standard_normal(case.N).astype(np.float16)
    say(f"[y only] {case.name} M={case.M} K={case.K} N={case.N} r={case.r} seed={case.seed} "
        f"bias={bias is not None} {kw}")
    g = run_gpu(X, W, want_acc=False, bias=bias, **kw)
    o = orc.linear(X, W, threshold=kw["threshold"], e=kw["e"], r_cap=kw["r_cap"],
                   w_gran=kw["w_gran"], rows=rows, bias16=bias, x_gran=kw.get("x_gran", "tensor"),
                   ia_bits=kw.get("ia_bits", 8), w_bits=kw.get("w_bits", 8))
    sel = slice(None) if rows is None else np.asarray(rows)
    assert g["n_outliers"].tolist() == [o["n_used"], o["n_total"]], f"{case.name}: n_outliers"
    tol = Y_REL_TOL * float(np.abs(o["y32"]).max())
    err = float(np.abs(g["Y"][sel].astype(np.float32) - o["y32"]).max())
    assert err <= tol, f"{case.name}: Y max abs err {err} > {tol}"
    same = g["Y"][sel] == o["y16"]
    assert same.all(), f"{case.name}: Y not bit-identical to the oracle ({(~same).sum()} elements)"
    return g, o


def sample_rows(M, n, seed, tile=256):
    rng = np.random.default_rng(seed)
    rows = set([0, M - 1, min(M - 1, tile - 1), min(M - 1, tile), (M // tile) * tile - 1 if M >= tile else 0])
    while len(rows) < min(n, M):
        rows.add(int(rng.integers(0, M)))
    return sorted(rows)


def rows_every_block(M, seed, block=64):
    """One row out of every `block` consecutive rows (a wave of the GEMM owns 64 rows of a
    256-row tile, so every tile and every wave position of every tile is sampled), plus the
    first and last row."""
    rng = np.random.default_rng(seed)
    rows = {0, M - 1}
    for b0 in range(0, M, block):
        rows.add(int(b0 + rng.integers(0, min(block, M - b0))))
    return sorted(rows)


def check_own_scale(case: synth.Case, X=None, W=None, bias_seed=None, **over):
    """muxq_linear with Aux on a scale of its own against the oracle's aux_scale="own": scales and
    codes bit for bit; the accumulators equal acc_body + rne(rho * acc_aux) with
    rho = (2^e - 1) s_aux / s_x in binary32 (the library's stated recombination); Y within half a
    unit of s_x s_w[n] plus rounding of the oracle's sum after dequantisation."""
    if X is None:
        X, W, _ = synth.make_case(case)
    kw = dict(w_gran=case.w_gran, threshold=case.threshold, e=case.exp, r_cap=case.r_cap)
    kw.update(over)
    bias = None
    if bias_seed is not None:
        bias = np.random.default_rng(bias_seed).standard_normal(W.shape[1]).astype(np.float16)
    say(f"[own-scale aux] {case.name} M={X.shape[0]} K={X.shape[1]} N={W.shape[1]} {kw} bias={bias is not None}")
    x_gran = kw.get("x_gran", "tensor")
    g = run_gpu(X, W, bias=bias, aux_scale="own", **kw)
    o = orc.linear(X, W, threshold=kw["threshold"], e=kw["e"], r_cap=kw["r_cap"], w_gran=kw["w_gran"],
                   bias16=bias, aux_scale="own", x_gran=x_gran)
    M, K, r, e = X.shape[0], X.shape[1], o["n_used"], kw["e"]
    assert g["n_outliers"].tolist() == [r, o["n_total"]]
    cfac = np.float32((1 << e) - 1)
    if x_gran == "tensor":
        assert g["x_scale"][0] == o["s_x"][0] and g["x_scale"][1] == o["inv_x"][0]
        if r:
            assert g["aux_scale"][0] == o["s_aux"][0] and g["aux_scale"][1] == o["inv_aux"][0], "s_aux"
        sx, sa = np.float32(o["s_x"][0]), np.float32(o["s_aux"][0])
        rho = (cfac * sa) / sx if sx > 0 else np.float32(0)
        sxc, sac, rhoc = float(sx), float(sa), rho
    else:
        assert (g["x_scale"][0] == o["s_x"]).all() and (g["x_scale"][1] == o["inv_x"]).all(), "token scales"
        sx, sa = o["s_x"].astype(np.float32), o["s_aux"].astype(np.float32)
        with np.errstate(divide="ignore", invalid="ignore"):
            rho = np.where(sx > 0, (cfac * sa) / sx, np.float32(0)).astype(np.float32)
        if r:
            assert (g["aux_scale"][0] == sa).all(), "s_aux per token"
            assert (g["aux_scale"][1] == rho).all(), "rho per token"
        sxc, sac, rhoc = sx.astype(np.float64).reshape(-1, 1), sa.astype(np.float64).reshape(-1, 1), rho.reshape(-1, 1)
    assert (g["body_q"][:, :K] == o["body_q"]).all(), "body_q"
    assert (g["aux_q"][:, :r] == o["aux_q"]).all() and (g["aux_q"][:, r:] == 0).all(), "aux_q"
    want = o["acc_body"].astype(np.int64) + np.rint(rhoc * o["acc_aux"].astype(np.float32)).astype(np.int64)
    assert (g["acc"] == want).all(), "accumulators after the rescale"
    sw = o["s_w"].astype(np.float64).reshape(1, -1)
    yg = g["Y"].astype(np.float64)
    # half a unit of s_x s_w[n] from rounding the Aux term to Body's grid; the fp16 rounding of
    # the output (2^-11 |y|); binary32 roundings of the two products on either side, which are
    # relative to the terms and not to their (possibly cancelling) sum
    c = float((1 << e) - 1)
    terms = np.abs(sxc * sw * o["acc_body"]) + np.abs(c * sac * sw * o["acc_aux"])
    tol = 0.5 * sxc * sw + 2.0 ** -10 * np.abs(o["y32"]) + 2.0 ** -20 * terms + 1e-30
    bad = np.abs(yg - o["y32"]) > tol
    assert not bad.any(), f"{case.name}: {bad.sum()} outputs beyond half a unit of s_x s_w"
    assert np.abs(yg - o["y32"]).max() <= Y_REL_TOL * float(np.abs(o["y32"]).max())
    return g, o


def check_mlp(M, K, N1, N2, seed, *, w_gran="tensor", x_gran="tensor", r=6, r_cap=64, e=2):
    """c_fc -> GELU -> c_proj (Sec. IV-C).  The fused first layer (GELU in the GEMM's epilogue,
    column maxima handed to the second layer) against (1) the unfused chain of the library's own
    entry points, bit for bit, and (2) the oracle: first-layer output before the GELU bit-exact,
    GELU within one fp16 unit in the last place on under 1 % of the elements, second layer stage
    by stage on the hidden activation the GPU produced."""
    dev = "cuda"
    rng = np.random.default_rng(seed)
    X, _ = synth.make_x(M, K, r, (20.0, 100.0), rng)
    W1 = synth.make_w(K, N1, rng)
    W2 = synth.make_w(N1, N2, rng)
    b1 = (0.5 * rng.standard_normal(N1)).astype(np.float16)
    b2 = (0.1 * rng.standard_normal(N2)).astype(np.float16)
    say(f"[mlp] M={M} {K}->{N1}->{N2} seed={seed} w={w_gran} x={x_gran}")
    Xd = torch.from_numpy(X).to(dev)
    wq1, ws1 = B.muxq_quantize_weight(torch.from_numpy(W1).to(dev), w_gran)
    wq2, ws2 = B.muxq_quantize_weight(torch.from_numpy(W2).to(dev), w_gran)
    b1d, b2d = torch.from_numpy(b1).to(dev), torch.from_numpy(b2).to(dev)
    kw = dict(threshold=6.0, exp=e, r_cap=r_cap, x_gran=x_gran)
    lay2 = B.workspace_layout(M, N1, N2, r_cap)
    # unfused: layer, stand-alone GELU (which leaves the maxima), layer
    wsa = B.alloc_workspace(M, N1, N2, r_cap)
    wsa.fill_(0xCD)
    Y1 = B.muxq_linear(Xd, wq1, ws1, N1, w_gran, bias=b1d, **kw)
    H_ref = B.muxq_gelu_absmax(Y1, wsa, lay2)
    Y2_ref = B.muxq_linear(H_ref, wq2, ws2, N2, w_gran, bias=b2d, workspace=wsa, absmax_ready=True, **kw)
    # fused
    wsb = B.alloc_workspace(M, N1, N2, r_cap)
    wsb.fill_(0xCD)
    H, n_slabs = B.muxq_linear_gelu(Xd, wq1, ws1, N1, w_gran, bias=b1d, next_workspace=wsb, next_layout=lay2, **kw)
    Y2 = B.muxq_linear(H, wq2, ws2, N2, w_gran, bias=b2d, workspace=wsb, absmax_ready=True,
                       absmax_slabs=n_slabs, **kw)
    torch.cuda.synchronize()
    assert 1 <= n_slabs <= 64
    assert torch.equal(H, H_ref), "fused GELU differs from the stand-alone GELU kernel"
    assert torch.equal(Y2, Y2_ref), "second layer differs"
    get = lambda ws, name: B.ws_view(ws, lay2, name, M, N2, r_cap).cpu().numpy()
    Hn = H.cpu().numpy()
    colmax = np.abs(Hn.astype(np.float32)).max(axis=0)
    assert (get(wsb, "col_absmax")[:N1] == colmax).all(), "column maxima handed over by the GEMM"
    # oracle, first layer and GELU
    o1 = orc.linear(X, W1, bias16=b1, w_gran=w_gran, x_gran=x_gran, e=e, r_cap=r_cap)
    assert (Y1.cpu().numpy() == o1["y16"]).all(), "first layer"
    g = orc.gelu_tanh(o1["y16"])
    diff = Hn != g
    ulp_apart = np.abs(Hn.view(np.int16).astype(np.int32) - g.view(np.int16).astype(np.int32))
    assert diff.mean() < 0.01 and ulp_apart[diff].max(initial=0) <= 1, "GELU beyond one unit in the last place"
    # oracle, second layer on the hidden activation the GPU produced
    o2 = orc.linear(Hn, W2, bias16=b2, w_gran=w_gran, x_gran=x_gran, e=e, r_cap=r_cap)
    assert get(wsb, "n_outliers").tolist() == [o2["n_used"], o2["n_total"]]
    assert (get(wsb, "outlier_idx")[:r_cap] == o2["outlier_idx"]).all()
    assert (Y2.cpu().numpy() == o2["y16"]).all(), "second layer against the oracle"
    # the block as one call: same H, same Y, the second layer's workspace behind the first's
    Hb, Yb, wsm = B.muxq_mlp(Xd, wq1, ws1, N1, wq2, ws2, N2, w_gran, bias1=b1d, bias2=b2d, **kw)
    torch.cuda.synchronize()
    assert torch.equal(Hb, H) and torch.equal(Yb, Y2), "muxq_mlp differs from its two calls"
    off2 = (B.workspace_layout(M, K, N1, r_cap).total + 255) // 256 * 256
    for name in ("n_outliers", "outlier_idx", "x_scale_token" if x_gran == "token" else "x_scale"):
        a = B.ws_view(wsm[off2:], lay2, name, M, N2, r_cap)
        b = B.ws_view(wsb, lay2, name, M, N2, r_cap)
        assert torch.equal(a, b), f"muxq_mlp: second layer's {name}"
    return n_slabs
