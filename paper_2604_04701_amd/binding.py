"""Thin ctypes binding of libmuxq.so (the C ABI declared in include/muxq.h).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the computation runs inside the library's kernels.
There is no CPU fallback: if the shared library is missing, loading raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmuxq.so")

PER_TENSOR, PER_CHANNEL = 0, 1
_GRAN = {"tensor": PER_TENSOR, "channel": PER_CHANNEL, PER_TENSOR: PER_TENSOR,
         PER_CHANNEL: PER_CHANNEL}

EXPORTS = ["muxq_version", "muxq_status_string", "muxq_k_pad", "muxq_wq_bytes",
           "muxq_packed_bytes", "muxq_packed_index", "muxq_detect_scratch_bytes",
           "muxq_workspace_layout", "muxq_workspace_bytes", "muxq_quantize_weight", "muxq_quantize_weight_bits", "muxq_linear_opts",
           "muxq_detect_outliers", "muxq_build_aux", "muxq_linear",
           "muxq_linear_naive_int8", "muxq_gemm_i8", "muxq_init", "muxq_linear_timed",
           "muxq_noalloc_max_bytes", "muxq_linear_noalloc", "muxq_linear_gelu", "muxq_linear_gelu_slabs",
           "muxq_mlp", "muxq_mlp_workspace_bytes",
           "muxq_quantize_weight_smooth", "muxq_smooth_absmax",
           "muxq_probe_mfma_rate", "muxq_static_bytes", "muxq_static_layout_of",
           "muxq_prepare_static", "muxq_linear_static", "muxq_gelu_absmax"]


class MuxqError(RuntimeError):
    pass


class WsLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in
                ("col_absmax", "col_scale", "col_slot", "col_mask", "outlier_idx", "n_outliers",
                 "x_scale", "absmax_partial", "body_q", "aux_q", "w_aux", "cn", "total")] + [("k_pad", C.c_int32)]


class StaticLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("col_mask", "outlier_idx", "n_outliers", "w_aux", "total")] + \
               [("k_pad", C.c_int32)]


class ActOpts(C.Structure):
    _fields_ = [("x_gran", C.c_int32), ("ia_bits", C.c_int32), ("absmax_ready", C.c_int32),
                ("aux_own_scale", C.c_int32), ("absmax_slabs", C.c_int32)]


X_PER_TENSOR, X_PER_TOKEN = 0, 1
_XGRAN = {"tensor": X_PER_TENSOR, "token": X_PER_TOKEN, X_PER_TENSOR: X_PER_TENSOR,
          X_PER_TOKEN: X_PER_TOKEN}

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MuxqError(f"{LIB_PATH} is missing: build it with "
                            "`python -m paper_2604_04701_amd.build` (there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i, f, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
        L.muxq_version.restype = i
        L.muxq_status_string.restype = C.c_char_p
        L.muxq_status_string.argtypes = [i]
        L.muxq_k_pad.restype = i
        L.muxq_k_pad.argtypes = [i]
        L.muxq_wq_bytes.restype = sz
        L.muxq_wq_bytes.argtypes = [i, i]
        L.muxq_packed_bytes.restype = sz
        L.muxq_packed_bytes.argtypes = [i, i]
        L.muxq_packed_index.restype = sz
        L.muxq_packed_index.argtypes = [i, i, i]
        L.muxq_workspace_layout.restype = i
        L.muxq_workspace_layout.argtypes = [i, i, i, i, C.POINTER(WsLayout)]
        L.muxq_workspace_bytes.restype = sz
        L.muxq_workspace_bytes.argtypes = [i, i, i, i]
        L.muxq_quantize_weight.restype = i
        L.muxq_quantize_weight.argtypes = [vp, i, i, i, i, vp, vp, vp]
        L.muxq_detect_outliers.restype = i
        L.muxq_detect_outliers.argtypes = [vp, i, i, i, f, i, vp, vp, vp, vp, vp]
        L.muxq_detect_scratch_bytes.restype = sz
        L.muxq_detect_scratch_bytes.argtypes = [i]
        L.muxq_build_aux.restype = i
        L.muxq_build_aux.argtypes = [vp, i, i, i, vp, vp, vp, i, i, vp, vp, vp, vp, vp]
        L.muxq_linear.restype = i
        L.muxq_linear.argtypes = [vp, i, i, i, vp, vp, i, i, vp, f, i, i, vp, i, vp, sz, vp, vp]
        L.muxq_quantize_weight_bits.restype = i
        L.muxq_quantize_weight_bits.argtypes = [vp, i, i, i, i, i, vp, vp, vp]
        L.muxq_linear_opts.restype = i
        L.muxq_linear_opts.argtypes = [vp, i, i, i, vp, vp, i, i, vp, f, i, i, vp, i, vp, sz, vp,
                                       C.POINTER(ActOpts), vp]
        L.muxq_linear_naive_int8.restype = i
        L.muxq_linear_naive_int8.argtypes = [vp, i, i, i, vp, vp, i, i, vp, vp, i, vp, sz, vp, vp]
        L.muxq_gemm_i8.restype = i
        L.muxq_gemm_i8.argtypes = [vp, i, i, vp, i, vp, vp, vp, i, i, vp, vp, i, vp, vp, i, vp, vp]
        L.muxq_probe_mfma_rate.restype = i
        L.muxq_probe_mfma_rate.argtypes = [vp, vp, sz, i, i, vp, vp]
        L.muxq_init.restype = i
        L.muxq_init.argtypes = []
        L.muxq_mlp_workspace_bytes.restype = sz
        L.muxq_mlp_workspace_bytes.argtypes = [i, i, i, i, i]
        L.muxq_mlp.restype = i
        L.muxq_mlp.argtypes = [vp, i, i, i, vp, vp, i, i, vp, vp, vp, i, i, vp, f, i, i, vp, i, vp, i, vp, sz,
                               C.POINTER(ActOpts), vp]
        L.muxq_noalloc_max_bytes.restype = sz
        L.muxq_noalloc_max_bytes.argtypes = []
        L.muxq_linear_noalloc.restype = i
        L.muxq_linear_noalloc.argtypes = [vp, i, i, i, vp, vp, i, i, vp, f, i, i, vp, i, vp]
        L.muxq_linear_timed.restype = i
        L.muxq_linear_timed.argtypes = [vp, i, i, i, vp, vp, i, i, vp, f, i, i, vp, i, vp, sz,
                                        C.POINTER(ActOpts), vp, vp, vp, vp]
        L.muxq_static_bytes.restype = sz
        L.muxq_static_bytes.argtypes = [i, i, i]
        L.muxq_static_layout_of.restype = i
        L.muxq_static_layout_of.argtypes = [i, i, i, C.POINTER(StaticLayout)]
        L.muxq_prepare_static.restype = i
        L.muxq_prepare_static.argtypes = [vp, i, i, vp, i, i, vp, sz, vp]
        L.muxq_linear_static.restype = i
        L.muxq_linear_static.argtypes = [vp, i, i, i, vp, vp, i, i, vp, i, i, vp, vp, i, vp, sz, vp,
                                         C.POINTER(ActOpts), vp]
        L.muxq_gelu_absmax.restype = i
        L.muxq_gelu_absmax.argtypes = [vp, i, i, i, vp, i, vp, vp]
        L.muxq_quantize_weight_smooth.restype = i
        L.muxq_quantize_weight_smooth.argtypes = [vp, i, i, i, i, i, vp, vp, vp, vp]
        L.muxq_smooth_absmax.restype = i
        L.muxq_smooth_absmax.argtypes = [vp, i, i, i, vp, vp, i, vp, vp]
        L.muxq_linear_gelu_slabs.restype = i
        L.muxq_linear_gelu_slabs.argtypes = [i, i, i]
        L.muxq_linear_gelu.restype = i
        L.muxq_linear_gelu.argtypes = [vp, i, i, i, vp, vp, i, i, vp, f, i, i, vp, i, vp, sz, vp,
                                       C.POINTER(ActOpts), vp]
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != 0:
        raise MuxqError(f"{what}: status {status} ({lib().muxq_status_string(status).decode()})")


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def k_pad(K: int) -> int:
    return lib().muxq_k_pad(K)


def packed_bytes(rows: int, cols: int) -> int:
    return lib().muxq_packed_bytes(rows, cols)


def unpack(buf, rows: int, cols: int):
    """Packed layout (16 x 64 blocks, see include/muxq.h) -> row-major [rows, cols] tensor.
    Pure re-indexing for tests and inspection; works on any device."""
    if cols == 0:
        return buf.new_empty((rows, 0))
    r16 = (rows + 15) // 16
    v = buf.reshape(-1)[:r16 * 16 * cols].view(r16, cols // 64, 16, 64)
    return v.permute(0, 2, 1, 3).reshape(r16 * 16, cols)[:rows]


def pack(mat):
    """Row-major [rows, cols] int8 tensor (cols % 64 == 0) -> packed flat buffer."""
    rows, cols = mat.shape
    r16 = (rows + 15) // 16
    full = mat.new_zeros((r16 * 16, cols))
    full[:rows] = mat
    return full.view(r16, 16, cols // 64, 64).permute(0, 2, 1, 3).contiguous().reshape(-1)


def workspace_layout(M, K, N, r_cap) -> WsLayout:
    L = WsLayout()
    _check(lib().muxq_workspace_layout(M, K, N, r_cap, C.byref(L)), "muxq_workspace_layout")
    return L


def workspace_bytes(M, K, N, r_cap) -> int:
    return lib().muxq_workspace_bytes(M, K, N, r_cap)


def alloc_workspace(M, K, N, r_cap, device="cuda"):
    return torch.empty(workspace_bytes(M, K, N, r_cap), dtype=torch.uint8, device=device)


def muxq_quantize_weight(W, gran="tensor", bits=8, factors=None):
    """W: [K, N] fp16 device tensor (row stride W.stride(0)).  Returns (w_q: packed
    N x k_pad int8 codes as a flat buffer, w_scale [1] or [N] fp32).  factors: optional fp32 [K]
    device tensor, the weight side of a per-channel difficulty migration (W' = fp16(W f[k]))."""
    K, N = W.shape
    g = _GRAN[gran]
    w_q = torch.empty(lib().muxq_wq_bytes(K, N), dtype=torch.int8, device=W.device)
    w_scale = torch.empty(N if g == PER_CHANNEL else 1, dtype=torch.float32, device=W.device)
    if factors is not None:
        _check(lib().muxq_quantize_weight_smooth(_p(W), K, N, W.stride(0), g, bits, _p(factors), _p(w_q),
                                                 _p(w_scale), _stream()), "muxq_quantize_weight_smooth")
    elif bits == 8:
        _check(lib().muxq_quantize_weight(_p(W), K, N, W.stride(0), g, _p(w_q), _p(w_scale),
                                          _stream()), "muxq_quantize_weight")
    else:
        _check(lib().muxq_quantize_weight_bits(_p(W), K, N, W.stride(0), g, bits, _p(w_q),
                                               _p(w_scale), _stream()), "muxq_quantize_weight_bits")
    return w_q, w_scale


def muxq_detect_outliers(X, threshold=6.0, r_cap=64):
    """Returns (col_absmax [K] fp32, outlier_idx [max(r_cap,1)] int32, n_outliers [2] int32)."""
    M, K = X.shape
    col_absmax = torch.empty(K, dtype=torch.float32, device=X.device)
    idx = torch.empty(max(r_cap, 1), dtype=torch.int32, device=X.device)
    n_out = torch.empty(2, dtype=torch.int32, device=X.device)
    scratch = torch.empty(lib().muxq_detect_scratch_bytes(K), dtype=torch.uint8, device=X.device)
    _check(lib().muxq_detect_outliers(_p(X), M, K, X.stride(0), threshold, r_cap, _p(col_absmax),
                                      _p(idx), _p(n_out), _p(scratch), _stream()),
           "muxq_detect_outliers")
    return col_absmax, idx, n_out


def muxq_build_aux(X, col_absmax, outlier_idx, n_outliers, r_cap=64, exp=2):
    """Returns (body_q packed M x k_pad, aux_q packed M x r_cap, x_scale [2] fp32)."""
    M, K = X.shape
    kp = k_pad(K)
    body_q = torch.empty(packed_bytes(M, kp), dtype=torch.int8, device=X.device)
    aux_q = torch.empty(packed_bytes(M, r_cap), dtype=torch.int8, device=X.device)
    x_scale = torch.empty(2, dtype=torch.float32, device=X.device)
    scratch = torch.empty(2 * kp, dtype=torch.int32, device=X.device)
    _check(lib().muxq_build_aux(_p(X), M, K, X.stride(0), _p(col_absmax), _p(outlier_idx),
                                _p(n_outliers), r_cap, exp, _p(body_q),
                                _p(aux_q) if r_cap else None, _p(x_scale), _p(scratch), _stream()),
           "muxq_build_aux")
    return body_q, aux_q, x_scale


def muxq_smooth_absmax(X, factors, workspace=None, layout=None, out=None):
    """X' = fp16(X / factors[k]) (in place when out is X); with workspace / layout also the slab
    maxima of X' for a following call with absmax_ready=True.  Returns X'."""
    M, K = X.shape
    if out is None:
        out = torch.empty_like(X)
    slabs = None if workspace is None else workspace[layout.absmax_partial:]
    _check(lib().muxq_smooth_absmax(_p(X), M, K, X.stride(0), _p(factors), _p(out), out.stride(0),
                                    _p(slabs), _stream()), "muxq_smooth_absmax")
    return out


def muxq_gelu_absmax(Y, workspace, layout: "WsLayout", out=None):
    """X = gelu(Y) (tanh form; in place when out is Y) and the slab maxima of X, left in the
    absmax_partial region of `workspace` (a muxq_linear workspace for the same M, K; `layout`
    its workspace_layout) for a following call with absmax_ready=True.  Returns X."""
    M, K = Y.shape
    if out is None:
        out = torch.empty_like(Y)
    slabs = workspace[layout.absmax_partial:]
    _check(lib().muxq_gelu_absmax(_p(Y), M, K, Y.stride(0), _p(out), out.stride(0), _p(slabs), _stream()),
           "muxq_gelu_absmax")
    return out


def muxq_linear(X, w_q, w_scale, N, w_gran="tensor", bias=None, threshold=6.0, exp=2, r_cap=64,
                out=None, workspace=None, dbg_acc=None, x_gran="tensor", ia_bits=8, absmax_ready=False,
                aux_scale="shared", absmax_slabs=0):
    """Y = MUXQ(X) . W.  X [M, K] fp16; w_q / w_scale from muxq_quantize_weight of a
    K x N weight.  Returns Y [M, N] fp16 (and leaves every intermediate in `workspace`).
    x_gran "token" / ia_bits != 8 / absmax_ready (slab maxima left in `workspace` by
    muxq_gelu_absmax) go through muxq_linear_opts."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(M, K, N, r_cap, X.device)
    own = {"shared": 0, "own": 1}[aux_scale]
    if _XGRAN[x_gran] == X_PER_TENSOR and ia_bits == 8 and not absmax_ready and not own and not absmax_slabs:
        _check(lib().muxq_linear(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran], N,
                                 _p(bias), threshold, exp, r_cap, _p(out), out.stride(0),
                                 _p(workspace), workspace.numel(), _p(dbg_acc), _stream()),
               "muxq_linear")
    else:
        opts = ActOpts(_XGRAN[x_gran], ia_bits, int(bool(absmax_ready)), own, absmax_slabs)
        _check(lib().muxq_linear_opts(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran],
                                      N, _p(bias), threshold, exp, r_cap, _p(out), out.stride(0),
                                      _p(workspace), workspace.numel(), _p(dbg_acc), C.byref(opts),
                                      _stream()), "muxq_linear_opts")
    return out


def muxq_linear_noalloc(X, w_q, w_scale, N, w_gran="tensor", bias=None, threshold=6.0, exp=2, r_cap=64,
                        out=None):
    """muxq_linear with its intermediates in the library's static device array (no workspace,
    no allocation inside the call; `out` is the caller's, allocated here only when not given)."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    _check(lib().muxq_linear_noalloc(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran], N,
                                     _p(bias), threshold, exp, r_cap, _p(out), out.stride(0), _stream()),
           "muxq_linear_noalloc")
    return out


def muxq_linear_gelu(X, w_q, w_scale, N, w_gran="tensor", bias=None, threshold=6.0, exp=2, r_cap=64,
                     out=None, workspace=None, next_workspace=None, next_layout=None, x_gran="tensor",
                     ia_bits=8):
    """H = gelu(MUXQ(X) . W + b) with the GELU fused into the GEMM.  next_workspace / next_layout:
    the workspace (and its workspace_layout) of the layer that consumes H; it receives H's slab
    maxima.  Returns (H, number of slabs written -- pass it on as absmax_slabs with
    absmax_ready=True)."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(M, K, N, r_cap, X.device)
    slabs = None if next_workspace is None else next_workspace[next_layout.absmax_partial:]
    opts = ActOpts(_XGRAN[x_gran], ia_bits, 0, 0, 0)
    _check(lib().muxq_linear_gelu(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran], N,
                                  _p(bias), threshold, exp, r_cap, _p(out), out.stride(0), _p(workspace),
                                  workspace.numel(), _p(slabs), C.byref(opts), _stream()),
           "muxq_linear_gelu")
    return out, lib().muxq_linear_gelu_slabs(M, K, N)


def muxq_mlp(X, w1_q, w1_scale, N1, w2_q, w2_scale, N2, w_gran="tensor", bias1=None, bias2=None,
             threshold=6.0, exp=2, r_cap=64, x_gran="tensor", ia_bits=8, workspace=None, out_h=None, out=None):
    """c_fc, GELU, c_proj as one call: returns (H, Y, workspace).  The workspace holds the first
    layer's workspace at offset 0 and the second layer's behind it (see muxq.h)."""
    M, K = X.shape
    if out_h is None:
        out_h = torch.empty((M, N1), dtype=torch.float16, device=X.device)
    if out is None:
        out = torch.empty((M, N2), dtype=torch.float16, device=X.device)
    if workspace is None:
        n = lib().muxq_mlp_workspace_bytes(M, K, N1, N2, r_cap)
        if n == 0:
            raise MuxqError("muxq_mlp_workspace_bytes: bad shapes")
        workspace = torch.empty(n, dtype=torch.uint8, device=X.device)
    opts = ActOpts(_XGRAN[x_gran], ia_bits, 0, 0, 0)
    _check(lib().muxq_mlp(_p(X), M, K, X.stride(0), _p(w1_q), _p(w1_scale), _GRAN[w_gran], N1, _p(bias1),
                          _p(w2_q), _p(w2_scale), _GRAN[w_gran], N2, _p(bias2), threshold, exp, r_cap,
                          _p(out_h), out_h.stride(0), _p(out), out.stride(0), _p(workspace),
                          workspace.numel(), C.byref(opts), _stream()), "muxq_mlp")
    return out_h, out, workspace


def static_layout(K, N, r_cap) -> StaticLayout:
    lay = StaticLayout()
    _check(lib().muxq_static_layout_of(K, N, r_cap, C.byref(lay)), "muxq_static_layout_of")
    return lay


def muxq_prepare_static(channel_list, K, w_q, N, r_cap=64):
    """channel_list: int32 tensor on the GPU (ascending channel indices found offline), may be
    empty.  Returns the static block (uint8 tensor) muxq_linear_static consumes."""
    lay = static_layout(K, N, r_cap)
    block = torch.empty(lay.total, dtype=torch.uint8, device=w_q.device)
    n = int(channel_list.numel())
    _check(lib().muxq_prepare_static(_p(channel_list) if n else None, n, K, _p(w_q), N, r_cap,
                                     _p(block), block.numel(), _stream()), "muxq_prepare_static")
    return block


def muxq_linear_static(X, w_q, w_scale, N, static_block, w_gran="tensor", bias=None, exp=2, r_cap=64,
                       out=None, workspace=None, dbg_acc=None, x_gran="tensor", ia_bits=8,
                       absmax_ready=False, aux_scale="shared", absmax_slabs=0):
    """muxq_linear with the channel list of a prepared static block instead of the run-time
    detection (per-token activations then need one pass over X)."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(M, K, N, r_cap, X.device)
    opts = ActOpts(_XGRAN[x_gran], ia_bits, int(bool(absmax_ready)), {"shared": 0, "own": 1}[aux_scale],
                   absmax_slabs)
    _check(lib().muxq_linear_static(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran], N,
                                    _p(bias), exp, r_cap, _p(static_block), _p(out), out.stride(0),
                                    _p(workspace), workspace.numel(), _p(dbg_acc), C.byref(opts),
                                    _stream()), "muxq_linear_static")
    return out


def muxq_linear_naive_int8(X, w_q, w_scale, N, w_gran="tensor", bias=None, out=None,
                           workspace=None, dbg_acc=None):
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(M, K, N, 0, X.device)
    _check(lib().muxq_linear_naive_int8(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale),
                                        _GRAN[w_gran], N, _p(bias), _p(out), out.stride(0),
                                        _p(workspace), workspace.numel(), _p(dbg_acc), _stream()),
           "muxq_linear_naive_int8")
    return out


def muxq_gemm_i8(a_q, M, K, w_q, N, x_scale, w_scale, w_gran="tensor", aux_q=None, w_aux=None,
                 n_outliers=None, r_cap=0, exp=2, bias=None, out=None, dbg_acc=None):
    """a_q / w_q / aux_q / w_aux: packed buffers (see pack / unpack)."""
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_q.device)
    _check(lib().muxq_gemm_i8(_p(a_q), M, K, _p(w_q), N, _p(aux_q), _p(w_aux),
                              _p(n_outliers), r_cap, exp, _p(x_scale), _p(w_scale), _GRAN[w_gran],
                              _p(bias), _p(out), out.stride(0), _p(dbg_acc), _stream()),
           "muxq_gemm_i8")
    return out


def muxq_init():
    """Per-device set-up for the current device (optional; needed before a first call that is
    made under graph capture)."""
    _check(lib().muxq_init(), "muxq_init")


def muxq_linear_timed(X, w_q, w_scale, N, gemm_start, gemm_stop, w_gran="tensor", bias=None,
                      threshold=6.0, exp=2, r_cap=64, out=None, workspace=None, x_gran="tensor",
                      ia_bits=8, absmax_ready=False, wg_ticks=None):
    """muxq_linear that records the raw hipEvent_t handles gemm_start / gemm_stop (ints) around
    its GEMM kernel (measurement aid, include/muxq_measure.h).  wg_ticks: None or an int64
    device tensor of 2048 entries (start / end tick of each workgroup of a persistent GEMM)."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(M, K, N, r_cap, X.device)
    opts = ActOpts(_XGRAN[x_gran], ia_bits, int(bool(absmax_ready)), 0)
    _check(lib().muxq_linear_timed(_p(X), M, K, X.stride(0), _p(w_q), _p(w_scale), _GRAN[w_gran], N,
                                   _p(bias), threshold, exp, r_cap, _p(out), out.stride(0),
                                   _p(workspace), workspace.numel(), C.byref(opts), gemm_start,
                                   gemm_stop, _p(wg_ticks), _stream()), "muxq_linear_timed")
    return out


def wq_row_sums(w_q, K: int, N: int):
    """The int32 per-output-channel code sums stored behind the packed codes of a weight."""
    off = (packed_bytes(N, k_pad(K)) + 255) // 256 * 256
    return w_q[off:off + 4 * N].view(torch.int32)


def ws_packed(workspace, layout: WsLayout, name: str, M: int, N: int, r_cap: int):
    """The raw packed buffer of body_q / aux_q / w_aux inside a muxq_linear workspace."""
    rows, cols = {"body_q": (M, layout.k_pad), "aux_q": (M, r_cap), "w_aux": (N, r_cap)}[name]
    off = getattr(layout, name)
    return workspace[off:off + packed_bytes(rows, cols)].view(torch.int8)


def ws_view(workspace, layout: WsLayout, name: str, M: int, N: int, r_cap: int):
    """Typed view of one intermediate inside a muxq_linear workspace (the three INT8
    matrices are returned unpacked to row-major)."""
    kp = layout.k_pad
    spec = {
        "col_absmax": (torch.float32, (kp,)),
        "col_scale": (torch.float32, (kp,)),
        "col_slot": (torch.int32, (kp,)),
        "outlier_idx": (torch.int32, (max(r_cap, 1),)),
        "n_outliers": (torch.int32, (2,)),
        "zero_point": (torch.int32, (1,)),
        "zero_point_token": (torch.int32, (M,)),
        "cn": (torch.int32, (N,)),
        "x_scale": (torch.float32, (2,)),
        "aux_scale": (torch.float32, (2,)),
        "x_scale_token": (torch.float32, (2, M)),
        "aux_scale_token": (torch.float32, (2, M)),      # s_aux[M], rho[M] (Aux on its own scale)
        "body_q": (torch.int8, (M, kp)),
        "aux_q": (torch.int8, (M, r_cap)),
        "w_aux": (torch.int8, (N, r_cap)),
    }[name]
    dtype, shape = spec
    if name in ("body_q", "aux_q", "w_aux"):
        off = getattr(layout, name)
        return unpack(workspace[off:off + packed_bytes(*shape)].view(torch.int8), *shape)
    n = 1
    for d in shape:
        n *= d
    if name == "zero_point":
        off = layout.n_outliers + 8
    elif name == "aux_scale":
        off = layout.x_scale + 8
    elif name == "aux_scale_token":
        off = layout.x_scale + 12 * M
    elif name == "zero_point_token":
        off = layout.x_scale + 8 * M
    else:
        off = getattr(layout, "x_scale" if name == "x_scale_token" else name)
    nbytes = n * torch.empty(0, dtype=dtype).element_size()
    return workspace[off:off + nbytes].view(dtype).view(shape)


def muxq_probe_mfma_rate(a_codes, b_codes, iters=4000, n_workgroups=512):
    """Register-only MFMA issue-rate probe on the given operand codes (int8 device tensors).
    Returns (TOP/s, shader GHz)."""
    n = min(a_codes.numel(), b_codes.numel()) // 16 * 16
    clocks = torch.zeros(3, dtype=torch.int64, device=a_codes.device)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    _check(lib().muxq_probe_mfma_rate(_p(a_codes), _p(b_codes), n, iters, n_workgroups, _p(clocks),
                                      _stream()), "muxq_probe_mfma_rate")
    stop.record()
    torch.cuda.synchronize()
    ops = n_workgroups * 4 * iters * 8 * 65536.0
    c = clocks.cpu().tolist()
    return ops / (start.elapsed_time(stop) * 1e-3) / 1e12, (c[0] / (c[1] * 10.0) if c[1] else 0.0)
