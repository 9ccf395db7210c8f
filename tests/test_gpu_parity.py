"""GPU parity: the HIP library against the CPU oracle, stage by stage, through
the C ABI.  INT8 codes, scales, outlier lists and INT32 accumulators must be
bit-exact; Y within 1e-2 * max|Y_fp32| (and, with the fixed op order, equal)."""
import numpy as np
import pytest
import torch

from gpu_common import check_mlp, check_own_scale, rows_every_block, check_case, check_plain_y, compare, run_gpu, sample_rows, say
from oracle import muxq_oracle as orc
from paper_2604_04701_amd import binding as B
from paper_2604_04701_amd import synth
from paper_2604_04701_amd.synth import Case

pytestmark = pytest.mark.gpu
U = (20.0, 100.0)


def test_config1_all_stages():
    check_case(synth.config_cases(1)[0])


@pytest.mark.parametrize("case", [
    Case("one_by_one_tile", 1, 8, 8, 1, U, 21),
    Case("ragged_small", 333, 200, 264, 3, U, 22),
    Case("ragged_k_tail", 70, 1032, 520, 5, U, 23),
    Case("tall_thin", 2049, 64, 8, 2, U, 24),
    Case("wide", 5, 512, 4104, 4, U, 25),
    Case("several_tiles", 777, 320, 1096, 7, U, 26),
], ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_ragged_shapes(case, w_gran):
    check_case(case, w_gran=w_gran, bias_seed=case.seed)


# Shapes with at least 192 tiles of 256 x 256: these take the persistent large-tile GEMM
# (several tiles per workgroup, ragged last tile row and column, one- and two-step K loops).
LARGE = [
    Case("large_ragged", 3333, 200, 4104, 5, U, 27),
    Case("large_k64", 4096, 64, 4096, 2, U, 28),
    Case("large_ragged_long", 2100, 712, 6152, 9, U, 29),
]


@pytest.mark.parametrize("case", LARGE, ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_large_tile_path_all_stages(case, w_gran):
    check_case(case, w_gran=w_gran, bias_seed=case.seed)


@pytest.mark.parametrize("case", LARGE, ids=lambda c: c.name)
@pytest.mark.parametrize("r_cap", [64, 0])
def test_large_tile_path_plain_epilogue(case, r_cap):
    # per-tensor scale, no bias, no accumulator export: the epilogue variant the benchmark runs
    check_plain_y(case, r_cap=r_cap)


@pytest.mark.parametrize("e", [0, 1, 2, 3, 7])
def test_exp_factors(e):
    check_case(Case("exp", 300, 256, 136, 6, U, 30 + e), e=e)


@pytest.mark.parametrize("r_cap,r", [(0, 5), (64, 0), (64, 64), (64, 70), (128, 100), (256, 3)])
def test_outlier_capacity(r_cap, r):
    # r_cap = 0 -> naive; fewer, exactly as many and more outlier channels than capacity
    check_case(Case("rcap", 260, 512, 264, r, U, 40 + r), r_cap=r_cap)


def test_degenerate_inputs():
    rng = np.random.default_rng(50)
    W = (rng.standard_normal((64, 72)) * 0.02).astype(np.float16)
    W[:, 3] = 0                                             # zero weight column (per-channel)
    X = np.zeros((40, 64), np.float16)                      # all-zero activations
    for gran in ("tensor", "channel"):
        g = run_gpu(X, W, w_gran=gran)
        o = orc.linear(X, W, w_gran=gran)
        compare(g, o, 64, 72, 64, what="zero X " + gran)
        assert np.isfinite(g["Y"]).all() and (g["Y"] == 0).all()
    X = rng.standard_normal((40, 64)).astype(np.float16)
    X[0, 0] = 6.0                                           # exactly the threshold: not an outlier
    X[1, 1] = np.float16(6.004)                             # next fp16 above 6: outlier
    X[:, 5] = 0
    X[2, 7] = np.float16(6e-8)                              # subnormal
    g = run_gpu(X, W, w_gran="channel")
    o = orc.linear(X, W, w_gran="channel")
    compare(g, o, 64, 72, 64, what="threshold edge")
    assert o["outlier_idx"][:o["n_used"]].tolist() == [1]
    Wz = np.zeros_like(W)
    g = run_gpu(X, Wz)
    o = orc.linear(X, Wz)
    compare(g, o, 64, 72, 64, what="zero W")


def test_non_finite_inputs_are_harmless():
    # the header promises unspecified codes but no fault for NaN / Inf in X: nothing the
    # kernels index with depends on a data value.  A NaN alone leaves every other channel's
    # handling intact (abs-max and threshold compare ignore it); the calls return, and the
    # next ordinary call is right.
    case = Case("nonfinite", 200, 256, 136, 4, U, 71)
    X, W, _ = synth.make_case(case)
    Xn = X.copy()
    Xn[17, 33] = np.float16("nan")
    for x_gran in ("tensor", "token"):
        g = run_gpu(Xn, W, x_gran=x_gran, finite=False)
        o = orc.linear(X, W, x_gran=x_gran)
        assert g["n_outliers"].tolist() == [o["n_used"], o["n_total"]]
        rows = [m for m in range(case.M) if m != 17]
        assert (g["body_q"][rows][:, :case.K] == o["body_q"][rows]).all()
    Xi = X.copy()
    Xi[3, 5] = np.float16("inf")
    Xi[9, 200] = -np.float16("inf")
    for x_gran in ("tensor", "token"):
        run_gpu(Xi, W, x_gran=x_gran, w_gran="channel", finite=False)          # must simply return
    check_case(case)


@pytest.mark.parametrize("x_gran", ["tensor", "token"])
def test_rounding_ties_with_a_zero_point(x_gran):
    # the zero point rides on the constant whose addition does the rounding: ties go to the
    # even SUM, so the zero point has to be even.  Half-integer Body values with scale 1
    # (an outlier channel whose shrunk maximum is exactly 127) and an odd largest unlisted code.
    rng = np.random.default_rng(5)
    M, K, N = 48, 64, 72
    X = (rng.integers(-9, 10, size=(M, K)) * 0.5).astype(np.float16)      # ..., -0.5, 0.5, 1.5, 2.5, ...
    X[:, 11] = 5.0 * np.sign(rng.standard_normal(M)).astype(np.float16)     # largest unlisted code: 5
    X[:, 7] = 508.0                                                         # listed; 508 / 4 = 127
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    g = run_gpu(X, W, x_gran=x_gran)
    o = orc.linear(X, W, x_gran=x_gran)
    assert o["n_used"] == 1 and float(o["inv_x"][0]) == 1.0
    assert np.all(np.asarray(g["zero_point"]) == 6)
    compare(g, o, K, N, 64, what="ties")


def test_accumulators_at_the_edge_of_int32():
    # every code at +-127 over a long K: |acc| = K * 127^2.  K = 133136 puts it 133 thousand below
    # 2^31, closer than the offset the accumulators start at (2^18 here: no zero point above
    # K = 65536), so the running sums pass through the wrap-around; integer arithmetic modulo
    # 2^32 must still give the exact accumulator.  K = 131072 is the longest row of the
    # per-token setting.
    # (r_cap = 0 there: the library refuses shapes whose worst-case |acc| exceeds INT32.)
    for K, r_cap, x_grans in ((133136, 0, ("tensor",)), (131072, 64, ("tensor", "token"))):
        M, N = 40, 72
        X = np.full((M, K), 4.0, dtype=np.float16)
        X[1::2] *= -1
        W = np.full((K, N), 0.001, dtype=np.float16)
        W[:, 1::3] *= -1
        for x_gran in x_grans:
            say(f"[edge] K={K} x={x_gran}")
            g = run_gpu(X, W, x_gran=x_gran, w_gran="channel", r_cap=r_cap)
            o = orc.linear(X, W, x_gran=x_gran, w_gran="channel", r_cap=r_cap)
            assert o["n_used"] == 0 and int(np.abs(o["acc"]).max()) == K * 127 * 127
            compare(g, o, K, N, r_cap, what=f"edge of int32, K={K}, {x_gran}")


def test_naive_entry_point_is_plain_int8():
    case = Case("naive", 300, 256, 264, 6, U, 60)
    X, W, _ = synth.make_case(case)
    g = run_gpu(X, W, naive=True)
    o = orc.linear(X, W, threshold=float("inf"), r_cap=0)
    compare(g, o, case.K, case.N, 0, what="naive")


def test_strided_inputs_and_outputs():
    case = Case("strided", 130, 128, 72, 3, U, 61)
    X, W, _ = synth.make_case(case)
    dev = "cuda"
    Xbig = torch.zeros((130, 160), dtype=torch.float16, device=dev)
    Xbig[:, :128] = torch.from_numpy(X).to(dev)
    Wbig = torch.zeros((128, 96), dtype=torch.float16, device=dev)
    Wbig[:, :72] = torch.from_numpy(W).to(dev)
    Ybig = torch.full((130, 88), 9.0, dtype=torch.float16, device=dev)
    w_q, w_scale = B.muxq_quantize_weight(Wbig[:, :72], "channel")
    Y = B.muxq_linear(Xbig[:, :128], w_q, w_scale, 72, "channel", out=Ybig[:, :72])
    torch.cuda.synchronize()
    o = orc.linear(X, W, w_gran="channel")
    assert (Y.cpu().numpy() == o["y16"]).all()
    assert (Ybig[:, 72:] == 9.0).all()                      # nothing written past N


def test_stage_entry_points():
    case = Case("stages", 515, 328, 72, 9, U, 62)
    X, W, _ = synth.make_case(case)
    Xd = torch.from_numpy(X).cuda()
    o = orc.linear(X, W, r_cap=64)
    col_absmax, idx, n_out = B.muxq_detect_outliers(Xd, 6.0, 64)
    body_q, aux_q, x_scale = B.muxq_build_aux(Xd, col_absmax, idx, n_out, 64, 2)
    torch.cuda.synchronize()
    assert (col_absmax.cpu().numpy() == o["col_absmax"]).all()
    assert (idx.cpu().numpy() == o["outlier_idx"]).all()
    assert n_out.cpu().tolist() == [o["n_used"], o["n_total"]]
    kp = B.k_pad(328)
    body_rm, aux_rm = B.unpack(body_q, 515, kp).cpu().numpy(), B.unpack(aux_q, 515, 64).cpu().numpy()
    assert (body_rm[:, :328] == o["body_q"]).all()
    assert (body_rm[:, 328:] == 0).all()
    assert (aux_rm[:, :o["n_used"]] == o["aux_q"]).all()
    assert (aux_rm[:, o["n_used"]:] == 0).all()
    assert x_scale.cpu().tolist() == [float(o["s_x"][0]), float(o["inv_x"][0])]
    # a caller-supplied (static) outlier list: the first three detected channels only
    n3 = torch.tensor([3, 3], dtype=torch.int32, device="cuda")
    body3, aux3, xs3 = B.muxq_build_aux(Xd, col_absmax, idx, n3, 64, 2)
    torch.cuda.synchronize()
    o3 = orc.linear(X, r_cap=3)
    assert (B.unpack(body3, 515, kp).cpu().numpy()[:, :328] == o3["body_q"]).all()
    assert (B.unpack(aux3, 515, 64).cpu().numpy()[:, :3] == o3["aux_q"]).all()
    assert xs3.cpu().tolist()[0] == float(o3["s_x"][0])
    # bare GEMM on those operands
    Wd = torch.from_numpy(W).cuda()
    w_q, w_scale = B.muxq_quantize_weight(Wd, "tensor")
    idx_np = o["outlier_idx"][:o["n_used"]]
    w_rm = B.unpack(w_q, 72, kp)
    w_aux_rm = torch.zeros((72, 64), dtype=torch.int8, device="cuda")
    w_aux_rm[:, :o["n_used"]] = w_rm[:, torch.from_numpy(idx_np.astype(np.int64)).cuda()]
    w_aux = B.pack(w_aux_rm)
    acc = torch.empty((515, 72), dtype=torch.int32, device="cuda")
    Y = B.muxq_gemm_i8(body_q, 515, 328, w_q, 72, x_scale, w_scale, "tensor", aux_q=aux_q,
                       w_aux=w_aux, n_outliers=n_out, r_cap=64, exp=2, dbg_acc=acc)
    torch.cuda.synchronize()
    assert (acc.cpu().numpy() == o["acc"]).all()
    assert (Y.cpu().numpy() == o["y16"]).all()
    Yb = B.muxq_gemm_i8(body_q, 515, 328, w_q, 72, x_scale, w_scale, "tensor", dbg_acc=acc)   # no Aux
    torch.cuda.synchronize()
    assert (acc.cpu().numpy() == o["acc_body"]).all()


def test_repeatable_and_workspace_reuse():
    case = Case("repeat", 600, 512, 520, 8, U, 63)
    X, W, _ = synth.make_case(case)
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda()
    w_q, w_scale = B.muxq_quantize_weight(Wd, "tensor")
    ws = B.alloc_workspace(600, 512, 520, 64)
    Y1 = B.muxq_linear(Xd, w_q, w_scale, 520, workspace=ws).clone()
    # a different input through the same workspace, then the first one again
    X2, _, _ = synth.make_case(Case("repeat2", 600, 512, 520, 30, U, 64))
    B.muxq_linear(torch.from_numpy(X2).cuda(), w_q, w_scale, 520, workspace=ws)
    Y3 = B.muxq_linear(Xd, w_q, w_scale, 520, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y3)
    assert (Y1.cpu().numpy() == orc.linear(X, W)["y16"]).all()


@pytest.mark.parametrize("case", synth.config_cases(2), ids=lambda c: c.name)
def test_config2(case):
    check_case(case)


# Full size: codes, scales and lists are compared over ALL rows; accumulators and Y on one row
# out of every 64 (every tile of the GEMM, every wave position inside every tile) ...
@pytest.mark.parametrize("case", synth.config_cases(3), ids=lambda c: c.name)
def test_config3_full_size_every_tile(case):
    check_case(case, rows=rows_every_block(case.M, case.seed))


@pytest.mark.parametrize("case", synth.config_cases(4), ids=lambda c: c.name)
def test_config4_full_size_every_tile(case):
    check_case(case, rows=rows_every_block(case.M, case.seed))


def test_config5_full_size_every_tile():
    case = synth.config_cases(5)[0]
    g, o = check_case(case, rows=rows_every_block(case.M, case.seed))
    assert o["n_used"] >= 32


# ... and over the whole matrix, every element, in the launch configuration bench.py times.
@pytest.mark.parametrize("case", [synth.config_cases(5)[0], synth.config_cases(4)[12],
                                  synth.config_cases(3)[4]], ids=lambda c: c.name)
def test_full_matrix_every_element(case):
    check_plain_y(case)


@pytest.mark.parametrize("case", [synth.config_cases(3)[2], synth.config_cases(4)[3],
                                  synth.config_cases(5)[0]], ids=lambda c: c.name)
def test_full_size_plain_epilogue_sampled_rows(case):
    # the launch configuration bench.py times: no accumulator export, no bias
    check_plain_y(case, rows=sample_rows(case.M, 32, case.seed + 1))


# ---- per-token activation scales (per-vector setting) and narrower code widths ----

TOKEN_CASES = [
    Case("tok_one", 1, 8, 8, 1, U, 71),
    Case("tok_ragged", 333, 200, 264, 3, U, 72),
    Case("tok_k_tail", 70, 1032, 520, 5, U, 73),
    Case("tok_k4096", 300, 4096, 136, 12, U, 74),
    Case("tok_k5120", 130, 5120, 72, 9, U, 75),           # 16 chunks per lane
    Case("tok_k7680", 24, 7680, 72, 6, U, 78),            # the longest rows kept in LDS (64 KiB per workgroup)
    Case("tok_k8704", 40, 8704, 72, 4, U, 76),            # rows read twice
]


@pytest.mark.parametrize("case", TOKEN_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_per_token_all_stages(case, w_gran):
    check_case(case, w_gran=w_gran, bias_seed=case.seed if w_gran == "channel" else None,
               x_gran="token")


def test_per_token_zero_rows_and_capacity():
    case = Case("tok_zero", 97, 256, 72, 70, U, 77)        # more outlier channels than capacity
    X, W, _ = synth.make_case(case)
    X[[0, 5, 96]] = 0                                        # all-zero tokens: scale 0, codes 0
    g = run_gpu(X, W, x_gran="token", w_gran="channel")
    o = orc.linear(X, W, x_gran="token", w_gran="channel")
    compare(g, o, case.K, case.N, 64, what="tok_zero")
    assert o["n_total"] > 64 and (g["Y"][[0, 5, 96]] == 0).all()


@pytest.mark.parametrize("case", [LARGE[0], LARGE[2]], ids=lambda c: c.name)
def test_per_token_large_tile_path(case):
    check_case(case, w_gran="channel", bias_seed=case.seed, x_gran="token")


@pytest.mark.parametrize("case", [synth.config_cases(3)[0], synth.config_cases(5)[0]],
                         ids=lambda c: c.name)
def test_per_token_full_size_sampled_rows(case):
    # the per-vector setting of Table 1: per-token activations with per-channel weights
    check_case(case, rows=sample_rows(case.M, 24, case.seed + 2), x_gran="token", w_gran="channel")


@pytest.mark.parametrize("ia_bits,w_bits", [(7, 8), (6, 8), (5, 8), (8, 5), (8, 4), (5, 4), (2, 2)])
@pytest.mark.parametrize("x_gran", ["tensor", "token"])
def test_bit_widths(ia_bits, w_bits, x_gran):
    case = Case("bits", 260, 512, 264, 6, U, 80 + ia_bits)
    check_case(case, w_gran="channel" if w_bits < 8 else "tensor", x_gran=x_gran,
               ia_bits=ia_bits, w_bits=w_bits)


def test_bit_widths_large_tile_path():
    check_case(LARGE[0], ia_bits=6, w_bits=5)
    check_case(LARGE[0], ia_bits=5, w_bits=8, x_gran="token", w_gran="channel")


# The large-tile GEMM fetches per-channel scales, bias and per-token scales into LDS with
# its first K step when no accumulator export is asked for: every combination, on exact and
# ragged tilings, with two-step and one-step K loops (K = 64 with and without Aux).
@pytest.mark.parametrize("case", LARGE, ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran,with_bias,x_gran", [
    ("channel", False, "tensor"), ("tensor", True, "tensor"), ("channel", True, "tensor"),
    ("tensor", False, "token"), ("channel", True, "token")])
def test_large_tile_path_staged_epilogue_constants(case, w_gran, with_bias, x_gran):
    check_plain_y(case, w_gran=w_gran, bias_seed=case.seed if with_bias else None, x_gran=x_gran)


def test_large_tile_path_staged_constants_one_step_tiles():
    check_plain_y(LARGE[1], w_gran="channel", bias_seed=5, r_cap=0)            # K = 64, no Aux
    check_plain_y(LARGE[1], w_gran="channel", bias_seed=6, x_gran="token", r_cap=0)


def test_config5_per_vector_with_bias_sampled_rows():
    case = synth.config_cases(5)[0]
    check_plain_y(case, rows=sample_rows(case.M, 24, 9), w_gran="channel", bias_seed=9, x_gran="token")


@pytest.mark.parametrize("r_cap,r", [(128, 100), (256, 130), (64, 90)])
def test_large_tile_path_several_aux_steps(r_cap, r):
    # two to three Aux K steps ahead of the Body steps, and a truncated list (r > r_cap)
    case = Case("large_aux", 3333, 512, 4104, r, U, 90 + r)
    check_case(case, r_cap=r_cap)
    check_plain_y(case, r_cap=r_cap, w_gran="channel", bias_seed=3)


# The 128 x 128 form of the DMA-ring GEMM: chosen below 144 tiles of 256 x 256 for long K
# loops (K >= 2048) and, with 1024 <= K < 2048, for 128..384 tiles of 128 x 128.  The third
# case (K = 64) runs the register-staged form on the same tiling.
MID = [
    Case("mid_long_k", 300, 2112, 264, 7, U, 41),
    Case("mid_one_round", 1500, 1032, 1544, 5, U, 42),
    Case("mid_k64", 1536, 64, 1536, 2, U, 43),
]


@pytest.mark.parametrize("case", MID, ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_mid_tile_path_all_stages(case, w_gran):
    check_case(case, w_gran=w_gran, bias_seed=case.seed)


@pytest.mark.parametrize("case", MID, ids=lambda c: c.name)
@pytest.mark.parametrize("w_gran,with_bias,x_gran,r_cap", [
    ("tensor", False, "tensor", 64), ("tensor", False, "tensor", 0), ("channel", False, "tensor", 64),
    ("tensor", True, "tensor", 64), ("tensor", False, "token", 64), ("channel", True, "token", 64),
    ("channel", True, "token", 0)])
def test_mid_tile_path_epilogue_forms(case, w_gran, with_bias, x_gran, r_cap):
    check_plain_y(case, w_gran=w_gran, bias_seed=case.seed if with_bias else None, x_gran=x_gran,
                  r_cap=r_cap)


@pytest.mark.parametrize("r_cap,r", [(128, 100), (256, 130), (64, 90)])
def test_mid_tile_path_several_aux_steps(r_cap, r):
    case = Case("mid_aux", 1500, 1088, 1544, r, U, 190 + r)
    check_case(case, r_cap=r_cap)
    check_plain_y(case, r_cap=r_cap, w_gran="channel", bias_seed=3)


def test_mid_tile_path_several_tiles_per_workgroup():
    # more 128 x 128 tiles than resident workgroups: the K-step stream runs across tiles
    case = Case("mid_stream", 2690, 2048, 3000, 9, U, 47)     # 132 tiles of 256^2, 528 of 128^2
    rows = sample_rows(case.M, 40, 11)
    check_case(case, rows=rows)
    check_plain_y(case, rows=rows)
    check_plain_y(case, rows=rows, w_gran="channel", bias_seed=4, x_gran="token")


def test_muxq_linear_recorded_in_a_graph_replays_correctly():
    # A call launches its four kernels on the given stream and nothing else (no allocation,
    # no memset, no host synchronisation), so it can be recorded into a HIP graph.  Every
    # replay, on fresh inputs and with eager work in between, must equal the eager call.
    import dataclasses
    case = Case("graph", 300, 256, 264, 5, U, 77)
    X, W, _ = synth.make_case(case)
    dev = "cuda"
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).to(dev), "channel")
    bias = np.random.default_rng(5).standard_normal(case.N).astype(np.float16)
    bd = torch.from_numpy(bias).to(dev)
    Xs = torch.from_numpy(X).to(dev)                       # the graph's input buffer
    ws = B.alloc_workspace(case.M, case.K, case.N, 64)
    Y = torch.empty((case.M, case.N), dtype=torch.float16, device=dev)

    def call():
        B.muxq_linear(Xs, w_q, w_scale, case.N, "channel", bias=bd, out=Y, workspace=ws)

    call()                                                 # first-use set-up happens outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        Xn, _, _ = synth.make_case(dataclasses.replace(case, seed=case.seed + 1 + rep, r=3 + 2 * rep))
        Xs.copy_(torch.from_numpy(Xn).to(dev))
        Y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        y_graph = Y.clone()
        Y.zero_()
        call()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, Y), f"replay {rep}"
        o = orc.linear(Xn, W, threshold=6.0, e=2, r_cap=64, w_gran="channel", bias16=bias)
        yg = y_graph.cpu().numpy().astype(np.float32)
        assert np.abs(yg - o["y32"]).max() <= 1e-2 * np.abs(o["y32"]).max(), f"replay {rep} vs oracle"


def test_accuracy_report_matches_the_oracle_route():
    # the SQNR table the library's report tool prints, against the oracle's evaluation
    # route (quantise, dequantise, fp64 product) on the same inputs: the GPU result is the
    # fp16 rounding of the same numbers, so the two figures agree closely, and MUXQ is
    # ahead of naive in every row
    from paper_2604_04701_amd import accuracy_report as R
    case = Case("acc", 256, 768, 512, 6, U, 3)
    X, W, _ = synth.make_case(case)
    rows = R.report(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda())
    assert len(rows) == len(R.WIDTHS) * len(R.GRANS)
    ref = X.astype(np.float64) @ W.astype(np.float64)
    for r in rows:
        kw = dict(x_gran=r["x_gran"], w_gran=r["w_gran"], ia_bits=r["ia_bits"], w_bits=r["w_bits"])
        m = orc.sqnr_db(orc.fake_quant_linear(X, W, muxq=True, **kw), ref)
        n = orc.sqnr_db(orc.fake_quant_linear(X, W, muxq=False, **kw), ref)
        assert r["outlier_channels"] == case.r
        assert abs(r["muxq_db"] - m) < 0.05 and abs(r["naive_db"] - n) < 0.05, (r, m, n)
        assert r["muxq_db"] > r["naive_db"]


@pytest.mark.timeout(900)
def test_packed_operand_beyond_two_gib():
    # Maximum sizes: the kernels address packed operands with 32-bit byte offsets, valid
    # below 4 GiB.  Here the Body codes take 2.2 GB, so offsets pass 2^31 (row 524288):
    # every stage must still match, including rows on both sides of that line.
    M, K, N = 540_008, 4096, 64
    rng = np.random.default_rng(123)
    block = rng.standard_normal((4096, K), dtype=np.float32)
    X = np.empty((M, K), np.float16)
    for i, r0 in enumerate(range(0, M, 4096)):
        n = min(4096, M - r0)
        X[r0:r0 + n] = (block[:n] * np.float32(0.6 + 0.1 * (i % 9))).astype(np.float16)
    cols = [7, 600, 1234, 3000, 4095]
    X[:, cols] = (X[:, cols].astype(np.float32) * 40.0).astype(np.float16)
    W = (rng.standard_normal((K, N), dtype=np.float32) * 0.02).astype(np.float16)
    line = (1 << 31) // K
    rows = sorted(set(sample_rows(M, 40, 5) + list(range(line - 20, line + 20)) + [M - 2, M - 1]))
    say(f"[max size] M={M} K={K} N={N}: packed Body {M * K / 2**30:.2f} GiB")
    g = run_gpu(X, W)
    o = orc.linear(X, W, rows=rows)
    compare(g, o, K, N, 64, rows=rows, what="beyond 2 GiB")
    del g, o
    g = run_gpu(X, W, x_gran="token", w_gran="channel")
    o = orc.linear(X, W, rows=rows, x_gran="token", w_gran="channel")
    compare(g, o, K, N, 64, rows=rows, what="beyond 2 GiB, per token")


def test_very_wide_output():
    # more Aux weight rows to gather than one grid dimension holds: the gather strides
    check_case(Case("wide_n", 16, 64, 300_000, 3, U, 61))
    check_plain_y(Case("wide_n_token", 24, 128, 280_000, 4, U, 62), x_gran="token", w_gran="channel",
                  bias_seed=2)


def _check_static(case, raw_list, x_gran, w_gran, r_cap=64, e=2, with_bias=False):
    """muxq_prepare_static + muxq_linear_static against the oracle run on the list the
    stated rule accepts (in range, strictly ascending)."""
    X, W, _ = synth.make_case(case)
    M, K, N = case.M, case.K, case.N
    accepted, prev = [], -1
    for k in raw_list:
        if prev < k < K:
            accepted.append(k)
            prev = k
    dev = "cuda"
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).to(dev), w_gran)
    block = B.muxq_prepare_static(torch.tensor(raw_list, dtype=torch.int32, device=dev), K, w_q, N, r_cap)
    ws = B.alloc_workspace(M, K, N, r_cap)
    ws.fill_(0xCD)
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev)
    bias = np.random.default_rng(8).standard_normal(N).astype(np.float16) if with_bias else None
    bd = torch.from_numpy(bias).to(dev) if with_bias else None
    say(f"[static] {case.name} M={M} K={K} N={N} list={len(raw_list)} accepted={len(accepted)} "
        f"x={x_gran} w={w_gran} r_cap={r_cap} e={e}")
    Y = B.muxq_linear_static(torch.from_numpy(X).to(dev), w_q, w_scale, N, block, w_gran, bias=bd, exp=e,
                             r_cap=r_cap, workspace=ws, dbg_acc=acc, x_gran=x_gran)
    torch.cuda.synchronize()
    o = orc.linear(X, W, e=e, r_cap=r_cap, w_gran=w_gran, x_gran=x_gran, bias16=bias, static_idx=accepted)
    r = o["n_used"]
    sl = B.static_layout(K, N, r_cap)
    idx_g = block[sl.outlier_idx:sl.outlier_idx + 4 * max(r_cap, 1)].view(torch.int32).cpu().numpy()
    n_g = block[sl.n_outliers:sl.n_outliers + 8].view(torch.int32).cpu().numpy()
    assert n_g.tolist() == [r, len(accepted)]
    if r_cap:
        assert (idx_g[:r_cap] == o["outlier_idx"]).all()
        w_aux = B.unpack(block[sl.w_aux:sl.w_aux + B.packed_bytes(N, r_cap)].view(torch.int8), N, r_cap)
        w_aux = w_aux.cpu().numpy()
        assert (w_aux[:, :r] == o["w_q"][o["outlier_idx"][:r], :].T).all() and (w_aux[:, r:] == 0).all()
    lay = B.workspace_layout(M, K, N, r_cap)
    get = lambda name: B.ws_view(ws, lay, name, M, N, r_cap).cpu().numpy()
    body_q = get("body_q").copy()
    unlisted = np.ones(K, bool)          # unlisted channels are stored as code + z
    unlisted[o["outlier_idx"][:r]] = False
    zrow = (get("zero_point_token") if x_gran == "token" else np.full(M, int(get("zero_point")[0]))).astype(np.int8)
    body_q[:, :K] -= zrow[:, None] * unlisted[None, :].astype(np.int8)
    wq_rows = B.unpack(w_q, N, lay.k_pad).cpu().numpy().astype(np.int64)[:, :K]
    # per-call zero point: cn carries the fixed offset that keeps the accumulators positive
    assert (get("cn") == wq_rows[:, unlisted].sum(axis=1) + ((1 << 14) if x_gran == "tensor" else 0)).all()
    assert (body_q[:, :K] == o["body_q"]).all() and (body_q[:, K:] == 0).all()
    if r_cap:
        aux_q = get("aux_q")
        assert (aux_q[:, :r] == o["aux_q"]).all() and (aux_q[:, r:] == 0).all()
    if x_gran == "token":
        xs = get("x_scale_token")
        assert (xs[0] == o["s_x"]).all() and (xs[1] == o["inv_x"]).all()
    else:
        xs = get("x_scale")
        assert xs[0] == o["s_x"][0] and xs[1] == o["inv_x"][0]
        assert (get("col_absmax")[:K] == o["col_absmax"]).all()
        assert get("n_outliers").tolist() == [r, r]      # the accepted count lives in the block
    assert (acc.cpu().numpy() == o["acc"]).all()
    yg = Y.cpu().numpy()
    assert ((yg == o["y16"]) | (np.isnan(yg) & np.isnan(o["y16"]))).all()


@pytest.mark.parametrize("x_gran,w_gran", [("tensor", "tensor"), ("token", "channel")])
def test_static_outlier_lists(x_gran, w_gran):
    case = Case("static", 300, 264, 136, 5, U, 81)
    _, _, planted = synth.make_case(case)
    planted = [int(k) for k in planted]
    # the list detection would find: the static call equals the dynamic one
    _check_static(case, planted, x_gran, w_gran)
    X, W, _ = synth.make_case(case)
    dyn = run_gpu(X, W, x_gran=x_gran, w_gran=w_gran)
    dev = "cuda"
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).to(dev), w_gran)
    block = B.muxq_prepare_static(torch.tensor(planted, dtype=torch.int32, device=dev), case.K, w_q, case.N)
    Y = B.muxq_linear_static(torch.from_numpy(X).to(dev), w_q, w_scale, case.N, block, w_gran, x_gran=x_gran)
    assert (Y.cpu().numpy() == dyn["Y"]).all()
    # a list that misses an outlier channel and names quiet ones; entries out of range,
    # repeated and out of order are skipped
    _check_static(case, [3, planted[0], planted[0], 2, 100, 263, 264, 9999, -4], x_gran, w_gran, with_bias=True)
    # empty list = naive; list longer than the capacity keeps the lowest entries
    _check_static(case, [], x_gran, w_gran)
    _check_static(case, list(range(0, 264, 2)), x_gran, w_gran, r_cap=64, e=3)
    _check_static(case, planted, x_gran, w_gran, r_cap=0)


@pytest.mark.parametrize("x_gran,w_gran", [("tensor", "tensor"), ("token", "channel")])
def test_static_outlier_lists_large_tile_path(x_gran, w_gran):
    case = LARGE[0]
    _, _, planted = synth.make_case(case)
    _check_static(case, [int(k) for k in planted] + [199], x_gran, w_gran, with_bias=True)
    case = Case("static_aux3", 3333, 512, 4104, 130, U, 83)
    _, _, planted = synth.make_case(case)
    _check_static(case, [int(k) for k in planted], x_gran, w_gran, r_cap=256)


def test_concurrent_calls_on_two_streams_with_their_own_workspaces():
    # calls that do not share a workspace may overlap: two streams (default priority), two
    # different problems, several rounds back to back; each result equals its solo run
    ca, cb = Case("stream_a", 700, 512, 776, 5, U, 91), LARGE[0]
    Xa, Wa, _ = synth.make_case(ca)
    Xb, Wb, _ = synth.make_case(cb)
    dev = "cuda"
    Xa_d, Xb_d = torch.from_numpy(Xa).to(dev), torch.from_numpy(Xb).to(dev)
    wqa, wsa = B.muxq_quantize_weight(torch.from_numpy(Wa).to(dev), "tensor")
    wqb, wsb = B.muxq_quantize_weight(torch.from_numpy(Wb).to(dev), "channel")
    ya_solo = B.muxq_linear(Xa_d, wqa, wsa, ca.N).clone()
    yb_solo = B.muxq_linear(Xb_d, wqb, wsb, cb.N, "channel", x_gran="token").clone()
    torch.cuda.synchronize()
    wsp_a = B.alloc_workspace(ca.M, ca.K, ca.N, 64)
    wsp_b = B.alloc_workspace(cb.M, cb.K, cb.N, 64)
    ya, yb = torch.empty_like(ya_solo), torch.empty_like(yb_solo)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(5):
        ya.zero_()
        yb.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            B.muxq_linear(Xa_d, wqa, wsa, ca.N, out=ya, workspace=wsp_a)
        with torch.cuda.stream(sb):
            B.muxq_linear(Xb_d, wqb, wsb, cb.N, "channel", out=yb, workspace=wsp_b, x_gran="token")
        torch.cuda.synchronize()
        assert torch.equal(ya, ya_solo) and torch.equal(yb, yb_solo)


# ---- producer fusion: GELU that leaves the slab maxima for the next layer ----

def _fp16_ulp_distance(a, b):
    """Distance in units of the last place between two fp16 arrays (finite values)."""
    def key(v):
        u = v.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a) - key(b))


@pytest.mark.parametrize("shape", [(1, 8), (333, 200), (70, 1032), (2049, 64), (1500, 4096)],
                         ids=lambda s: f"{s[0]}x{s[1]}")
def test_gelu_producer_matches_the_oracle_and_its_own_maxima(shape):
    M, K = shape
    rng = np.random.default_rng(M * 131 + K)
    Y = (rng.standard_normal((M, K)) * 2.5).astype(np.float16)
    Y[0, 0] = 0.0
    if M > 2:
        Y[1, :8] = np.array([-9.0, 9.0, -0.75, 6e-8, -6e-8, 65504.0, -65504.0, 0.5], dtype=np.float16)
        Y[2, K - 1] = 40.0                                       # a maximum in the last channel
    say(f"[gelu] M={M} K={K}")
    N, r_cap = 72, 64
    lay = B.workspace_layout(M, K, N, r_cap)
    ws = B.alloc_workspace(M, K, N, r_cap)
    Yd = torch.from_numpy(Y).cuda()
    Xd = B.muxq_gelu_absmax(Yd, ws, lay)
    X = Xd.cpu().numpy()
    want = orc.gelu_tanh(Y)
    d = _fp16_ulp_distance(X, want)
    # binary32 evaluation against the exact value rounded once: never more than one unit in the
    # last place apart, and that only where the exact value sits next to a rounding boundary
    assert d.max() <= 1 and (d != 0).mean() < 0.01, (int(d.max()), float((d != 0).mean()))
    # in place: the same bits
    Yd2 = Yd.clone()
    B.muxq_gelu_absmax(Yd2, ws, lay, out=Yd2)
    assert torch.equal(Yd2, Xd)
    # the maxima left in the workspace are those of X as written: the layer that starts from
    # them gives, bit for bit, what the layer that takes its own maxima gives
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).cuda(), "channel")
    for x_gran in ("tensor", "token"):
        B.muxq_gelu_absmax(Yd, ws, lay, out=Xd)
        y_fused = B.muxq_linear(Xd, w_q, w_scale, N, "channel", r_cap=r_cap, workspace=ws, x_gran=x_gran,
                                absmax_ready=True).clone()
        fused = {k: B.ws_view(ws, lay, k, M, N, r_cap).clone() for k in ("col_absmax", "outlier_idx", "n_outliers")}
        ws2 = B.alloc_workspace(M, K, N, r_cap)
        y_plain = B.muxq_linear(Xd, w_q, w_scale, N, "channel", r_cap=r_cap, workspace=ws2, x_gran=x_gran)
        assert torch.equal(y_fused, y_plain)
        for k, v in fused.items():
            # n_outliers[2] holds the per-call zero point, if any; col_absmax is K long inside k_pad
            n = {"n_outliers": 2, "col_absmax": K}.get(k, v.numel())
            assert torch.equal(v[:n], B.ws_view(ws2, lay, k, M, N, r_cap)[:n]), k
        o = orc.linear(X, W, w_gran="channel", x_gran=x_gran, r_cap=r_cap)
        assert (y_fused.cpu().numpy() == o["y16"]).all()
        assert (fused["col_absmax"].cpu().numpy()[:K] == o["col_absmax"]).all()
    # a static channel list with per-tensor activations still needs the maxima (for the scale)
    block = B.muxq_prepare_static(torch.tensor([0, K - 1], dtype=torch.int32, device="cuda"), K, w_q, N, r_cap)
    B.muxq_gelu_absmax(Yd, ws, lay, out=Xd)
    y_fused = B.muxq_linear_static(Xd, w_q, w_scale, N, block, "channel", r_cap=r_cap, workspace=ws,
                                   absmax_ready=True).clone()
    y_plain = B.muxq_linear_static(Xd, w_q, w_scale, N, block, "channel", r_cap=r_cap, workspace=ws2)
    assert torch.equal(y_fused, y_plain)
    o = orc.linear(X, W, w_gran="channel", r_cap=r_cap, static_idx=np.unique(np.array([0, K - 1], dtype=np.int32)))
    assert (y_fused.cpu().numpy() == o["y16"]).all()


def test_mfma_rate_probe_runs_and_reports_clocks():
    codes = torch.randint(-30, 31, (1 << 16,), dtype=torch.int8, device="cuda")
    tops, ghz = B.muxq_probe_mfma_rate(codes, codes, iters=200, n_workgroups=256)
    assert 100.0 < tops < 5500.0 and 0.5 < ghz < 3.0


# ---- Aux on a scale of its own (the other reading of Eq. 5) ----

def _barely_outlier_data(M, K, N, seed):
    """Outlier channels only just above the threshold: after the shift they are smaller than the
    normal channels, so Aux's own abs-max differs from Body's."""
    rng = np.random.default_rng(seed)
    X = rng.uniform(-5.0, 5.0, size=(M, K)).astype(np.float32)
    ch = np.sort(rng.choice(K, size=min(5, K // 4), replace=False))
    X[:, ch] = rng.uniform(-7.5, 7.5, size=(M, ch.size))
    X[0, ch] = 7.5
    W = (0.05 * rng.standard_normal((K, N))).astype(np.float16)
    return X.astype(np.float16), W


@pytest.mark.parametrize("shape", [(40, 64, 72), (333, 200, 264), (700, 1032, 520), (1500, 512, 1544),
                                   (2049, 2112, 1096)])
@pytest.mark.parametrize("e", [1, 2, 3])
def test_own_scale_aux_when_body_absmax_is_on_a_normal_channel(shape, e):
    M, K, N = shape
    X, W = _barely_outlier_data(M, K, N, 7 * M + e)
    case = Case(f"own_{M}x{K}x{N}", M, K, N, 5, U, 0)
    g, o = check_own_scale(case, X, W, e=e, w_gran="channel" if e == 2 else "tensor",
                           bias_seed=M if e == 3 else None)
    assert o["s_aux"][0] < o["s_x"][0] and np.abs(o["aux_q"]).max() == 127


@pytest.mark.parametrize("case", [Case("own_ragged_small", 333, 200, 264, 3, U, 22), LARGE[0],
                                  synth.config_cases(2)[3]], ids=lambda c: c.name)
def test_own_scale_aux_equals_the_shared_reading_on_loud_outliers(case):
    g, o = check_own_scale(case)
    assert o["s_aux"][0] == o["s_x"][0]
    X, W, _ = synth.make_case(case)
    shared = run_gpu(X, W, w_gran=case.w_gran, threshold=case.threshold, e=case.exp, r_cap=case.r_cap)
    assert (shared["aux_q"] == g["aux_q"]).all() and (shared["body_q"] == g["body_q"]).all()
    assert (shared["acc"] == g["acc"]).all()             # rho = 2^e - 1 exactly: same integers
    assert (shared["Y"] == g["Y"]).all()


def test_own_scale_aux_full_size_and_rejections():
    check_own_scale(synth.config_cases(3)[4])            # 8192 x 1024 -> 4096, the persistent kernel
    # no outlier channel at all, and capacity 0: the option changes nothing
    X, W, _ = synth.make_case(Case("own_none", 200, 128, 72, 0, U, 5))
    a = run_gpu(X, W, aux_scale="own")
    b = run_gpu(X, W)
    assert (a["Y"] == b["Y"]).all() and a["n_outliers"].tolist() == [0, 0]
    a = run_gpu(X, W, aux_scale="own", r_cap=0)
    assert (a["Y"] == b["Y"]).all()
    # the option is not combined with the fused GELU
    Xd = torch.from_numpy(X).cuda()
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).cuda(), "tensor")
    opts = B.ActOpts(0, 8, 0, 1, 0)
    H = torch.empty((200, 72), dtype=torch.float16, device="cuda")
    ws = B.alloc_workspace(200, 128, 72, 64)
    import ctypes as C
    st = B.lib().muxq_linear_gelu(Xd.data_ptr(), 200, 128, 128, w_q.data_ptr(), w_scale.data_ptr(), 0, 72, None,
                                  6.0, 2, 64, H.data_ptr(), 72, ws.data_ptr(), ws.numel(), None, C.byref(opts),
                                  None)
    assert st == 4


@pytest.mark.parametrize("shape", [(40, 64, 72), (333, 200, 264), (700, 1032, 520), (1500, 512, 1544),
                                   (2049, 2112, 1096), (3333, 200, 4104)])
@pytest.mark.parametrize("e", [1, 2, 3])
def test_own_scale_aux_with_one_scale_per_token(shape, e):
    """The per-vector setting with Aux on a scale of its own per token: scales, codes and the
    factors rho[m] bit for bit; accumulators acc_body + rne(rho[m] acc_aux); Y to the stated
    tolerance; and the call without the accumulator export (constants staged by the GEMM itself)
    gives the same Y as the call with it."""
    M, K, N = shape
    X, W = _barely_outlier_data(M, K, N, 11 * M + e)
    case = Case(f"own_tok_{M}x{K}x{N}", M, K, N, 5, U, 0)
    g, o = check_own_scale(case, X, W, e=e, w_gran="channel", x_gran="token",
                           bias_seed=M if e == 3 else None)
    assert (o["s_aux"] <= o["s_x"]).all() and (o["s_aux"] < o["s_x"]).any()
    assert (np.abs(o["aux_q"]).max(axis=1) == 127).all()          # every row's Aux uses its full range
    bias = np.random.default_rng(M).standard_normal(N).astype(np.float16) if e == 3 else None
    plain = run_gpu(X, W, w_gran="channel", x_gran="token", aux_scale="own", e=e, bias=bias, want_acc=False)
    assert (plain["Y"] == g["Y"]).all(), "with and without the accumulator export"


@pytest.mark.parametrize("x_gran,w_gran", [("tensor", "tensor"), ("token", "channel")])
def test_own_scale_aux_with_a_static_list(x_gran, w_gran):
    """A list fixed offline that names the channels detection would find, Aux on its own scale:
    the same result as the dynamic call (which is held to the oracle above)."""
    M, K, N = 700, 1032, 520
    X, W = _barely_outlier_data(M, K, N, 4242)
    dyn = run_gpu(X, W, w_gran=w_gran, x_gran=x_gran, aux_scale="own", want_acc=False)
    listed = [int(k) for k in dyn["outlier_idx"] if k >= 0]
    assert len(listed) == 5
    dev = "cuda"
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).to(dev), w_gran)
    block = B.muxq_prepare_static(torch.tensor(listed, dtype=torch.int32, device=dev), K, w_q, N)
    Y = B.muxq_linear_static(torch.from_numpy(X).to(dev), w_q, w_scale, N, block, w_gran, x_gran=x_gran,
                             aux_scale="own")
    assert (Y.cpu().numpy() == dyn["Y"]).all()


def test_own_scale_aux_per_token_full_size_and_loud_outliers():
    c = synth.config_cases(3)[5]                          # 8192 x 1024 -> 4096, per-channel weights
    X, W, _ = synth.make_case(c)
    g, o = check_own_scale(c, X, W, x_gran="token")
    # loud outliers: in most rows max|Body| sits on an outlier channel, s_aux[m] = s_x[m] there and
    # the rescale factor is 2^e - 1 exactly; such rows equal the shared reading bit for bit
    same = o["s_aux"] == o["s_x"]
    assert same.mean() > 0.9
    shared = run_gpu(X, W, w_gran=c.w_gran, x_gran="token", want_acc=False)
    assert (shared["Y"][same] == g["Y"][same]).all()


# ---- the MLP pair: GELU fused into the first projection's GEMM, maxima handed to the second ----

@pytest.mark.parametrize("shape,form", [
    ((3333, 200, 4104, 264), "persistent 256, ragged tiles"),
    ((1000, 2112, 1096, 520), "persistent 128"),
    ((300, 264, 520, 136), "register-staged: maxima by a pass over H"),
    ((2049, 512, 2048, 512), "register-staged 128"),
    ((4096, 64, 4096, 72), "persistent 256, one-step K loop"),
], ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
@pytest.mark.parametrize("w_gran,x_gran", [("tensor", "tensor"), ("channel", "token")])
def test_mlp_gelu_fused_into_the_first_gemm(shape, form, w_gran, x_gran):
    M, K, N1, N2 = shape
    check_mlp(M, K, N1, N2, seed=M + K, w_gran=w_gran, x_gran=x_gran)


def test_mlp_full_size_gpt2_medium():
    n = check_mlp(8192, 1024, 4096, 1024, seed=3100)       # configuration 3: c_fc, GELU, c_proj
    assert n == 32                                         # one slab per row of 256 x 256 tiles
    assert B.lib().muxq_linear_gelu_slabs(16384 * 2, 1024, 4096) == B.lib().muxq_linear_gelu_slabs(16384 * 2, 1024, 4096)
    # more than 64 rows of tiles: the maxima come from a pass over H, at that pass's slab count
    assert 1 <= B.lib().muxq_linear_gelu_slabs(32768, 1024, 4096) <= 64


# ---- per-channel difficulty migration (the combination Sec. V names) ----

@pytest.mark.parametrize("shape", [(333, 200, 264), (2049, 1032, 520), (1000, 4096, 1096)],
                         ids=lambda v: "x".join(map(str, v)))
@pytest.mark.parametrize("w_gran", ["tensor", "channel"])
def test_smoothing_combined_with_the_decomposition(shape, w_gran):
    M, K, N = shape
    case = Case(f"smooth_{M}", M, K, N, 7, (20.0, 60.0), 7000 + M)
    X, W, _ = synth.make_case(case)
    cx = np.abs(X.astype(np.float32)).max(axis=0)
    cw = np.abs(W.astype(np.float32)).max(axis=1)
    f = np.sqrt(np.maximum(cx, 1e-3) / np.maximum(cw, 1e-3)).astype(np.float32)
    f = (f / np.float32(np.median(f))).astype(np.float32)
    Xs, Ws = orc.smooth(X, W, f)                                     # the oracle's operands
    dev = "cuda"
    fd = torch.from_numpy(f).to(dev)
    Xd, Wd = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev)
    # weight side: codes of W' without materialising it
    w_q, w_scale = B.muxq_quantize_weight(Wd, w_gran, factors=fd)
    ow = orc.quantize_weight(Ws, w_gran)
    kp = B.k_pad(K)
    assert (B.unpack(w_q, N, kp)[:, :K].cpu().numpy() == ow["w_q"].T).all(), "codes of the smoothed weight"
    assert (w_scale.cpu().numpy() == ow["s_w"]).all()
    assert (B.wq_row_sums(w_q, K, N).cpu().numpy() == ow["w_q"].astype(np.int64).sum(axis=0)).all()
    # activation side: X' and its slab maxima, then the layer on them
    ws = B.alloc_workspace(M, K, N, 64)
    lay = B.workspace_layout(M, K, N, 64)
    ws.fill_(0xCD)
    Xsd = B.muxq_smooth_absmax(Xd, fd, ws, lay)
    assert (Xsd.cpu().numpy() == Xs).all(), "smoothed activations"
    Y = B.muxq_linear(Xsd, w_q, w_scale, N, w_gran, workspace=ws, absmax_ready=True)
    o = orc.linear(Xs, Ws, w_gran=w_gran)
    torch.cuda.synchronize()
    assert B.ws_view(ws, lay, "n_outliers", M, N, 64).tolist() == [o["n_used"], o["n_total"]]
    assert (B.ws_view(ws, lay, "col_absmax", M, N, 64)[:K].cpu().numpy() == o["col_absmax"]).all()
    assert (Y.cpu().numpy() == o["y16"]).all(), "layer on the smoothed operands"
    # in place, no maxima wanted
    X2 = Xd.clone()
    B.muxq_smooth_absmax(X2, fd, out=X2)
    assert torch.equal(X2, Xsd)
