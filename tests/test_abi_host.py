"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, sizes its buffers as documented, and turns bad
arguments into status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2604_04701_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000            # non-NULL, 256-byte aligned; never dereferenced on the error paths


def test_library_exports_every_declared_symbol():
    declared = set()
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        if not name.endswith(".h"):
            continue
        hdr = open(os.path.join(inc, name)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        declared |= set(re.findall(r"\b(muxq_[a-z0-9_]+)\s*\(", hdr))
    # the product header carries no measurement hook
    product = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "muxq.h")).read(), flags=re.S)
    assert "muxq_probe_mfma_rate" not in product and "muxq_linear_timed" not in product
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.muxq_version() >= 100
    assert L.muxq_status_string(0) == b"ok"
    for st in range(1, 7):
        assert len(L.muxq_status_string(st)) > 3


def test_sizes_and_layout():
    assert B.k_pad(768) == 768 and B.k_pad(8) == 64 and B.k_pad(200) == 256
    L = B.lib()
    up = lambda v: (v + 255) // 256 * 256
    assert L.muxq_wq_bytes(768, 2304) == 768 * 2304 + up(2304 * 4)     # codes, then int32 code sums
    assert L.muxq_wq_bytes(200, 264) == up(256 * 272) + up(264 * 4)    # rows padded to 16
    assert L.muxq_packed_bytes(17, 128) == 32 * 128 and L.muxq_packed_bytes(5, 100) == 0
    assert L.muxq_packed_index(0, 0, 128) == 0 and L.muxq_packed_index(1, 0, 128) == 64
    assert L.muxq_packed_index(0, 64, 128) == 1024 and L.muxq_packed_index(16, 5, 128) == 2048 + 5
    assert L.muxq_packed_index(17, 70, 128) == 2048 + 1024 + 64 + 6
    lay = B.workspace_layout(8192, 4096, 16384, 64)
    offs = [lay.col_absmax, lay.col_scale, lay.col_slot, lay.col_mask, lay.outlier_idx, lay.n_outliers,
            lay.x_scale, lay.absmax_partial, lay.body_q, lay.aux_q, lay.w_aux, lay.cn, lay.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lay.aux_q - lay.body_q >= 8192 * 4096
    assert lay.w_aux - lay.aux_q >= 8192 * 64
    assert lay.cn - lay.w_aux >= 16384 * 64 and lay.total - lay.cn >= 16384 * 4
    assert lay.total == B.workspace_bytes(8192, 4096, 16384, 64)
    # bad shapes -> 0 bytes / error status
    assert B.workspace_bytes(0, 768, 768, 64) == 0
    assert B.workspace_bytes(128, 770, 768, 64) == 0      # K % 8
    assert B.workspace_bytes(128, 768, 772, 64) == 0      # N % 8
    assert B.workspace_bytes(128, 768, 768, 32) == 0      # r_cap % 64
    assert B.workspace_bytes(128, 768, 768, 832) == 0     # r_cap > k_pad


def _linear(**kw):
    a = dict(X=FAKE, M=128, K=768, ldx=768, w_q=FAKE, w_scale=FAKE, w_gran=0, N=768, bias=None,
             threshold=6.0, exp=2, r_cap=64, Y=FAKE, ldy=768, ws=FAKE, ws_bytes=1 << 30, dbg=None,
             stream=None)
    a.update(kw)
    return B.lib().muxq_linear(a["X"], a["M"], a["K"], a["ldx"], a["w_q"], a["w_scale"],
                               a["w_gran"], a["N"], a["bias"], a["threshold"], a["exp"],
                               a["r_cap"], a["Y"], a["ldy"], a["ws"], a["ws_bytes"], a["dbg"],
                               a["stream"])


@pytest.mark.parametrize("kw,status", [
    (dict(X=None), 1), (dict(w_q=None), 1), (dict(Y=None), 1), (dict(ws=None), 1),
    (dict(M=0), 2), (dict(K=772), 2), (dict(N=100), 2), (dict(ldx=760), 2), (dict(ldy=764), 2),
    (dict(X=FAKE + 8), 3), (dict(ws=FAKE + 16), 3), (dict(Y=FAKE + 2), 3),
    (dict(exp=8), 4), (dict(exp=-1), 4), (dict(r_cap=65), 4), (dict(w_gran=2), 4),
    (dict(threshold=float("nan")), 4),
    (dict(ws_bytes=1000), 5),
])
def test_muxq_linear_rejects_bad_arguments(kw, status):
    assert _linear(**kw) == status


def test_other_entry_points_reject_bad_arguments():
    L = B.lib()
    assert L.muxq_quantize_weight(None, 768, 768, 768, 0, FAKE, FAKE, None) == 1
    assert L.muxq_quantize_weight(FAKE, 768, 768, 760, 0, FAKE, FAKE, None) == 2
    assert L.muxq_quantize_weight(FAKE, 768, 768, 768, 3, FAKE, FAKE, None) == 4
    assert L.muxq_detect_outliers(FAKE, 16, 768, 768, 6.0, 64, None, FAKE, FAKE, FAKE, None) == 1
    assert L.muxq_detect_outliers(FAKE, 16, 768, 768, 6.0, 64, FAKE, FAKE, FAKE, None, None) == 1
    assert L.muxq_detect_outliers(FAKE, 16, 768, 768, 6.0, 100, FAKE, FAKE, FAKE, FAKE, None) == 4
    assert L.muxq_detect_scratch_bytes(768) == 64 * 768 * 2
    assert L.muxq_build_aux(FAKE, 16, 768, 768, FAKE, FAKE, FAKE, 64, 2, FAKE, None, FAKE,
                            FAKE, None) == 1
    assert L.muxq_build_aux(FAKE, 16, 200, 192, FAKE, FAKE, FAKE, 64, 2, FAKE, FAKE, FAKE,
                            FAKE, None) == 2          # ldx < K
    assert L.muxq_gemm_i8(FAKE, 16, 768, FAKE, 768, FAKE, None, None, 64, 2, FAKE, FAKE, 0,
                          None, FAKE, 768, None, None) == 1   # partial aux operands
    assert L.muxq_gemm_i8(FAKE, 16, 768, FAKE, 768, None, None, None, 0, 2, FAKE, FAKE, 0,
                          None, FAKE, 760, None, None) == 2
    assert L.muxq_linear_naive_int8(FAKE, 16, 768, 768, FAKE, FAKE, 0, 768, None, FAKE, 768,
                                    FAKE, 10, None, None) == 5


def test_size_limits():
    big = 1 << 40
    assert _linear(N=(1 << 21) + 8, ldy=(1 << 21) + 8, ws_bytes=big) == 2
    assert _linear(K=(1 << 21) + 8, ldx=(1 << 21) + 8, ws_bytes=big) == 2
    assert _linear(M=(1 << 24) + 1, ws_bytes=big) == 2
    # packed Body of 4 GiB and more: 32-bit offsets no longer reach
    assert _linear(M=1 << 20, K=4096, ldx=4096, ws_bytes=big) == 2


def test_accumulator_overflow_guard():
    # 127^2 (K + (2^exp-1) r_cap) must stay below 2^31
    assert _linear(K=8 * 16384, ldx=8 * 16384, exp=7, r_cap=1024, ws_bytes=1 << 40) == 4


def _linear_opts(x_gran=0, ia_bits=8, **kw):
    a = dict(X=FAKE, M=128, K=768, ldx=768, w_q=FAKE, w_scale=FAKE, w_gran=0, N=768, bias=None,
             threshold=6.0, exp=2, r_cap=64, Y=FAKE, ldy=768, ws=FAKE, ws_bytes=1 << 30, dbg=None,
             stream=None)
    a.update(kw)
    opts = B.ActOpts(x_gran, ia_bits)
    import ctypes as C
    return B.lib().muxq_linear_opts(a["X"], a["M"], a["K"], a["ldx"], a["w_q"], a["w_scale"],
                                    a["w_gran"], a["N"], a["bias"], a["threshold"], a["exp"],
                                    a["r_cap"], a["Y"], a["ldy"], a["ws"], a["ws_bytes"], a["dbg"],
                                    C.byref(opts), a["stream"])


def test_option_entry_points_reject_bad_arguments():
    L = B.lib()
    assert _linear_opts(x_gran=2) == 4
    assert _linear_opts(ia_bits=1) == 4 and _linear_opts(ia_bits=9) == 4
    assert _linear_opts(x_gran=1, X=None) == 1                       # the usual checks still apply
    assert _linear_opts(x_gran=1, K=8192, ldx=8192, r_cap=8192, ws_bytes=1 << 40) == 4   # r_cap > 4096
    assert L.muxq_quantize_weight_bits(FAKE, 768, 768, 768, 0, 1, FAKE, FAKE, None) == 4
    assert L.muxq_quantize_weight_bits(FAKE, 768, 768, 768, 0, 9, FAKE, FAKE, None) == 4
    assert L.muxq_quantize_weight_bits(None, 768, 768, 768, 0, 4, FAKE, FAKE, None) == 1
    # the per-token setting needs room for two floats per row in the workspace
    lay_small, lay_big = B.workspace_layout(16, 768, 768, 64), B.workspace_layout(4096, 768, 768, 64)
    assert lay_big.absmax_partial - lay_big.x_scale >= 4096 * 12      # s_x, its reciprocal form, z
    assert lay_small.absmax_partial - lay_small.x_scale >= 16 * 12


def test_static_entry_points_reject_bad_arguments():
    L = B.lib()
    lay = B.static_layout(768, 2304, 64)
    offs = [lay.col_mask, lay.outlier_idx, lay.n_outliers, lay.w_aux, lay.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and lay.k_pad == 768
    assert lay.total - lay.w_aux >= 2304 * 64 and lay.total == L.muxq_static_bytes(768, 2304, 64)
    assert L.muxq_static_bytes(770, 2304, 64) == 0 and L.muxq_static_bytes(768, 2304, 32) == 0
    big = 1 << 30
    assert L.muxq_prepare_static(FAKE, 4, 768, None, 2304, 64, FAKE, big, None) == 1
    assert L.muxq_prepare_static(None, 4, 768, FAKE, 2304, 64, FAKE, big, None) == 1
    assert L.muxq_prepare_static(FAKE, -1, 768, FAKE, 2304, 64, FAKE, big, None) == 4
    assert L.muxq_prepare_static(FAKE, 4, 768, FAKE, 2304, 64, FAKE + 16, big, None) == 3
    assert L.muxq_prepare_static(FAKE, 4, 768, FAKE, 2304, 64, FAKE, 100, None) == 5
    opts = B.ActOpts(1, 8)
    args = lambda block: (FAKE, 128, 768, 768, FAKE, FAKE, 0, 768, None, 2, 64, block, FAKE, 768, FAKE,
                          big, None, C.byref(opts), None)
    assert L.muxq_linear_static(*args(None)) == 1
    assert L.muxq_linear_static(*args(FAKE + 8)) == 3
    bad = list(args(FAKE))
    bad[9] = 9                                     # exp out of range
    assert L.muxq_linear_static(*bad) == 4


def test_producer_fusion_entry_point_rejects_bad_arguments():
    L = B.lib()
    assert L.muxq_gelu_absmax(None, 16, 768, 768, FAKE, 768, FAKE, None) == 1
    assert L.muxq_gelu_absmax(FAKE, 16, 768, 768, None, 768, FAKE, None) == 1
    assert L.muxq_gelu_absmax(FAKE, 16, 768, 768, FAKE, 768, None, None) == 1
    assert L.muxq_gelu_absmax(FAKE, 16, 772, 776, FAKE, 776, FAKE, None) == 2      # K % 8
    assert L.muxq_gelu_absmax(FAKE, 16, 768, 760, FAKE, 768, FAKE, None) == 2      # ldy < K
    assert L.muxq_gelu_absmax(FAKE, 16, 768, 768, FAKE, 772, FAKE, None) == 2      # ldx % 8
    assert L.muxq_gelu_absmax(FAKE, 0, 768, 768, FAKE, 768, FAKE, None) == 2
    assert L.muxq_gelu_absmax(FAKE + 8, 16, 768, 768, FAKE, 768, FAKE, None) == 3
    assert L.muxq_gelu_absmax(FAKE, 16, 768, 768, FAKE, 768, FAKE + 4, None) == 3
    # the slab region of a workspace is the scratch of the detection entry point
    lay = B.workspace_layout(4096, 768, 768, 64)
    assert lay.body_q - lay.absmax_partial >= L.muxq_detect_scratch_bytes(768)


def test_mlp_entry_point_checks_both_layers_before_launching():
    """muxq_mlp validates the arguments of both layers before anything is launched (none of
    these calls reaches a kernel: there is no GPU here, and the pointers are fake)."""
    L = B.lib()
    M, K, N1, N2 = 256, 768, 3072, 768
    need = L.muxq_mlp_workspace_bytes(M, K, N1, N2, 64)
    l1, l2 = B.workspace_layout(M, K, N1, 64), B.workspace_layout(M, N1, N2, 64)
    assert need == (l1.total + 255) // 256 * 256 + l2.total
    assert L.muxq_mlp_workspace_bytes(M, 772, N1, N2, 64) == 0

    def call(**kw):
        a = dict(X=FAKE, M=M, K=K, ldx=K, w1=FAKE, s1=FAKE, g1=0, N1=N1, b1=None, w2=FAKE, s2=FAKE, g2=0,
                 N2=N2, b2=None, thr=6.0, exp=2, r_cap=64, H=FAKE, ldh=N1, Y=FAKE, ldy=N2, ws=FAKE, wsb=need,
                 opts=None)
        a.update(kw)
        return L.muxq_mlp(a["X"], a["M"], a["K"], a["ldx"], a["w1"], a["s1"], a["g1"], a["N1"], a["b1"],
                          a["w2"], a["s2"], a["g2"], a["N2"], a["b2"], a["thr"], a["exp"], a["r_cap"],
                          a["H"], a["ldh"], a["Y"], a["ldy"], a["ws"], a["wsb"], a["opts"], None)
    assert call(ws=None) == 1
    assert call(ws=FAKE + 16) == 3
    assert call(wsb=need - 1) == 5
    assert call(X=None) == 1                       # first layer
    assert call(ldx=K - 8) == 2
    assert call(w2=None) == 1                      # second layer, refused before the first is launched
    assert call(Y=None) == 1
    assert call(ldy=N2 - 8) == 2
    assert call(ldh=N1 - 8) == 2
    assert call(g2=7) == 4
    assert call(exp=9) == 4
    own = B.ActOpts(0, 8, 0, 1, 0)
    assert call(opts=C.byref(own)) == 4            # Aux on its own scale is not combined with the fused GELU


def test_noalloc_entry_point_refuses_oversize_before_touching_the_gpu():
    L = B.lib()
    assert L.muxq_noalloc_max_bytes() == 16 << 20
    assert B.workspace_bytes(8192, 4096, 16384, 64) > L.muxq_noalloc_max_bytes()
    st = L.muxq_linear_noalloc(FAKE, 8192, 4096, 4096, FAKE, FAKE, 0, 16384, None, 6.0, 2, 64, FAKE, 16384, None)
    assert st == 5                                           # MUXQ_ERR_WORKSPACE
    assert L.muxq_linear_noalloc(FAKE, 128, 772, 772, FAKE, FAKE, 0, 768, None, 6.0, 2, 64, FAKE, 768, None) == 2
