"""ctypes front end of the MUXQ CPU oracle -- TEST INFRASTRUCTURE ONLY.

Sequences the C steps of ``muxq_oracle.c`` in the order the paper gives them
(Sec. III-C Eq. 4-7 on top of the abs-max quantiser of Sec. II-A Eq. 1-3) and
returns every intermediate so tests can compare stage by stage.  numpy is used
for storage and for the two exact format conversions (fp16 -> fp32 widening of
the inputs, fp32 -> fp16 round-to-nearest-even of the output); all of the
method's arithmetic is in the C file.  The one exception is
``fake_quant_linear`` at the end: the evaluation procedure of Sec. IV-C
(quantise, dequantise, multiply in floating point), written out in numpy
fp64 as a second, independent route to the same layer output; and
``gelu_tanh``, the activation that sits between the two MLP projections of the
GPT-2 blocks the method is applied to (Sec. IV-C), written out in numpy fp64
for the producer-fusion entry points; ``mlp`` chains c_fc, that GELU and c_proj.
``linear`` carries two switches for readings the paper leaves open
(``aux_scale="own"``: Eq. 5 with an abs-max scale of Aux's own and Eq. 7 summed
after dequantisation; ``literal_div``: Eq. 1-2 with a division per element);
``smooth`` is the per-channel difficulty migration Sec. V says the method can be
combined with.

Nothing here imports or calls the GPU library, and the GPU library never
imports this module.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        f32p, i32p, i8p = (C.POINTER(C.c_float), C.POINTER(C.c_int32),
                           C.POINTER(C.c_int8))
        i64, i32, f32 = C.c_int64, C.c_int32, C.c_float
        sig = {
            "muxq_oracle_col_absmax": (None, [f32p, i64, i64, i64, f32p]),
            "muxq_oracle_select_outliers": (i32, [f32p, i64, f32, i32, i32p, i32p]),
            "muxq_oracle_decompose": (None, [f32p, i64, i64, i64, i32p, i32, i32, f32p, f32p]),
            "muxq_oracle_reconstruct": (None, [f32p, f32p, i64, i64, i32p, i32, i32, f32p]),
            "muxq_oracle_absmax": (f32, [f32p, i64]),
            "muxq_oracle_scale": (None, [f32, i32, f32p, f32p]),
            "muxq_oracle_quantize": (None, [f32p, i64, f32, i32, i8p]),
            "muxq_oracle_quantize_rows": (None, [f32p, i64, i64, f32p, i32, i8p]),
            "muxq_oracle_quantize_cols": (None, [f32p, i64, i64, f32p, i32, i8p]),
            "muxq_oracle_row_absmax": (None, [f32p, i64, i64, f32p]),
            "muxq_oracle_gather_rows": (None, [i8p, i64, i32p, i32, i8p]),
            "muxq_oracle_gemm_i8": (None, [i8p, i8p, i64, i64, i64, i32p]),
            "muxq_oracle_recombine": (None, [i32p, i32p, i64, i32, i32p]),
            "muxq_oracle_dequant": (None, [i32p, i64, i64, f32p, i32, f32p, i32, f32p, f32p]),
            "muxq_oracle_quantize_div": (None, [f32p, i64, i64, f32p, i64, i64, i32, i8p]),
            "muxq_oracle_dequant_sum": (None, [i32p, i32p, i64, i64, f32p, f32p, i32, f32p, i32, i32,
                                               f32p, f32p]),
            "muxq_oracle_scale_cols": (None, [f32p, i64, i64, f32p, i32, f32p]),
            "muxq_oracle_scale_rows": (None, [f32p, i64, i64, f32p, i32, f32p]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def n_threads() -> int:
    """Threads the OpenMP loops of the oracle use on this host."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def qmax_of(bits: int) -> int:
    """Largest code of a symmetric `bits`-bit integer grid, 2^(bits-1) - 1."""
    assert 2 <= bits <= 8
    return (1 << (bits - 1)) - 1


def _f32(a):
    """fp16 (or any float) array -> contiguous fp32, exact for fp16 input."""
    return np.ascontiguousarray(np.asarray(a).astype(np.float32))


# ---------------------------------------------------------------- stages ----

def col_absmax(X32):
    M, K = X32.shape
    out = np.empty(K, np.float32)
    lib().muxq_oracle_col_absmax(_ptr(X32, C.c_float), M, K, K, _ptr(out, C.c_float))
    return out


def select_outliers(colmax, threshold, r_cap):
    K = colmax.shape[0]
    idx = np.full(max(r_cap, 1), -1, np.int32)
    n_total = C.c_int32(0)
    n_used = lib().muxq_oracle_select_outliers(
        _ptr(colmax, C.c_float), K, C.c_float(threshold), r_cap,
        _ptr(idx, C.c_int32), C.byref(n_total))
    return idx[:r_cap], int(n_used), int(n_total.value)


def decompose(X32, idx, r, e):
    M, K = X32.shape
    body = np.empty((M, K), np.float32)
    aux = np.empty((M, max(r, 1)), np.float32)
    idxc = np.ascontiguousarray(idx[:max(r, 1)].astype(np.int32))
    lib().muxq_oracle_decompose(_ptr(X32, C.c_float), M, K, K, _ptr(idxc, C.c_int32),
                                r, e, _ptr(body, C.c_float), _ptr(aux, C.c_float))
    return body, aux[:, :r]


def reconstruct(body, aux, idx, r, e):
    M, K = body.shape
    auxc = np.ascontiguousarray(aux.reshape(M, r)) if r else np.zeros((M, 1), np.float32)
    out = np.empty((M, max(r, 1)), np.float32)
    idxc = np.ascontiguousarray(idx[:max(r, 1)].astype(np.int32))
    lib().muxq_oracle_reconstruct(_ptr(body, C.c_float), _ptr(auxc, C.c_float), M, K,
                                  _ptr(idxc, C.c_int32), r, e, _ptr(out, C.c_float))
    return out[:, :r]


def absmax(V32):
    V32 = np.ascontiguousarray(V32)
    return np.float32(lib().muxq_oracle_absmax(_ptr(V32, C.c_float), V32.size))


def scale(amax, qmax=127):
    s, inv = C.c_float(0), C.c_float(0)
    lib().muxq_oracle_scale(C.c_float(float(amax)), qmax, C.byref(s), C.byref(inv))
    return np.float32(s.value), np.float32(inv.value)


def quantize(V32, inv, qmax=127):
    V32 = np.ascontiguousarray(V32)
    q = np.empty(V32.shape, np.int8)
    lib().muxq_oracle_quantize(_ptr(V32, C.c_float), V32.size, C.c_float(float(inv)),
                               qmax, _ptr(q, C.c_int8))
    return q


def quantize_rows(V32, inv_row, qmax=127):
    V32 = np.ascontiguousarray(V32)
    inv_row = np.ascontiguousarray(inv_row, np.float32)
    q = np.empty(V32.shape, np.int8)
    lib().muxq_oracle_quantize_rows(_ptr(V32, C.c_float), V32.shape[0], V32.shape[1],
                                    _ptr(inv_row, C.c_float), qmax, _ptr(q, C.c_int8))
    return q


def quantize_cols(V32, inv_col, qmax=127):
    V32 = np.ascontiguousarray(V32)
    inv_col = np.ascontiguousarray(inv_col, np.float32)
    q = np.empty(V32.shape, np.int8)
    lib().muxq_oracle_quantize_cols(_ptr(V32, C.c_float), V32.shape[0], V32.shape[1],
                                    _ptr(inv_col, C.c_float), qmax, _ptr(q, C.c_int8))
    return q


def row_absmax(V32):
    V32 = np.ascontiguousarray(V32)
    out = np.empty(V32.shape[0], np.float32)
    lib().muxq_oracle_row_absmax(_ptr(V32, C.c_float), V32.shape[0], V32.shape[1],
                                 _ptr(out, C.c_float))
    return out


def gather_rows(wq, idx, r):
    K, N = wq.shape
    out = np.empty((max(r, 1), N), np.int8)
    idxc = np.ascontiguousarray(idx[:max(r, 1)].astype(np.int32))
    lib().muxq_oracle_gather_rows(_ptr(wq, C.c_int8), N, _ptr(idxc, C.c_int32), r,
                                  _ptr(out, C.c_int8))
    return out[:r]


def gemm_i8(A, B):
    A = np.ascontiguousarray(A, np.int8)
    B = np.ascontiguousarray(B, np.int8)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    if K == 0:
        acc[:] = 0
        return acc
    lib().muxq_oracle_gemm_i8(_ptr(A, C.c_int8), _ptr(B, C.c_int8), M, N, K,
                              _ptr(acc, C.c_int32))
    return acc


def recombine(acc_body, acc_aux, e):
    out = np.empty_like(acc_body)
    lib().muxq_oracle_recombine(_ptr(acc_body, C.c_int32), _ptr(acc_aux, C.c_int32),
                                acc_body.size, e, _ptr(out, C.c_int32))
    return out


def dequant(acc, s_x, s_w, bias32=None):
    M, N = acc.shape
    s_x = np.ascontiguousarray(np.atleast_1d(s_x), np.float32)
    s_w = np.ascontiguousarray(np.atleast_1d(s_w), np.float32)
    assert s_x.size in (1, M) and s_w.size in (1, N)
    y = np.empty((M, N), np.float32)
    bp = _ptr(bias32, C.c_float) if bias32 is not None else None
    lib().muxq_oracle_dequant(_ptr(acc, C.c_int32), M, N, _ptr(s_x, C.c_float),
                              int(s_x.size != 1),
                              _ptr(s_w, C.c_float), int(s_w.size != 1), bp,
                              _ptr(y, C.c_float))
    return y


def quantize_div(V32, s, per="tensor", qmax=127):
    """Eq. 1-2 read literally, q = round(v / s) with an fp32 division per element.
    per: "tensor" (s has one entry), "row" (one per row) or "col" (one per column)."""
    V32 = np.ascontiguousarray(V32, np.float32)
    rows, cols = V32.shape
    s = np.ascontiguousarray(np.atleast_1d(s), np.float32)
    assert s.size == {"tensor": 1, "row": rows, "col": cols}[per]
    q = np.empty(V32.shape, np.int8)
    lib().muxq_oracle_quantize_div(_ptr(V32, C.c_float), rows, cols, _ptr(s, C.c_float),
                                   int(per == "row"), int(per == "col"), qmax, _ptr(q, C.c_int8))
    return q


def dequant_sum(acc_body, acc_aux, s_x, s_aux, s_w, e, bias32=None):
    """Eq. 7 recombined after dequantisation (Aux on a scale of its own)."""
    M, N = acc_body.shape
    s_x = np.ascontiguousarray(np.atleast_1d(s_x), np.float32)
    s_aux = np.ascontiguousarray(np.atleast_1d(s_aux), np.float32)
    s_w = np.ascontiguousarray(np.atleast_1d(s_w), np.float32)
    assert s_x.size in (1, M) and s_aux.size == s_x.size and s_w.size in (1, N)
    y = np.empty((M, N), np.float32)
    bp = _ptr(bias32, C.c_float) if bias32 is not None else None
    lib().muxq_oracle_dequant_sum(_ptr(acc_body, C.c_int32), _ptr(acc_aux, C.c_int32), M, N,
                                  _ptr(s_x, C.c_float), _ptr(s_aux, C.c_float), int(s_x.size != 1),
                                  _ptr(s_w, C.c_float), int(s_w.size != 1), e, bp, _ptr(y, C.c_float))
    return y


def smooth(X16, W16, f):
    """Difficulty migration (the combination Sec. V names): X' = X diag(f)^-1, W' = diag(f) W
    with positive per-channel factors f (fp32), each computed in fp32 and rounded to fp16.
    The factors are an input: how they are chosen (e.g. max|X_k|^a / max|W_k|^(1-a) on
    calibration data) is outside the layer.  Returns (X' fp16, W' fp16)."""
    X32, W32 = _f32(X16), _f32(W16)
    f = np.ascontiguousarray(f, np.float32)
    M, K = X32.shape
    N = W32.shape[1]
    assert f.shape == (K,) and (f > 0).all()
    xo, wo = np.empty_like(X32), np.empty_like(W32)
    lib().muxq_oracle_scale_cols(_ptr(X32, C.c_float), M, K, _ptr(f, C.c_float), 1, _ptr(xo, C.c_float))
    lib().muxq_oracle_scale_rows(_ptr(W32, C.c_float), K, N, _ptr(f, C.c_float), 0, _ptr(wo, C.c_float))
    with np.errstate(over="ignore"):
        return xo.astype(np.float16), wo.astype(np.float16)


# ------------------------------------------------------------- sequences ----

def quantize_weight(W16, gran="tensor", bits=8, literal_div=False):
    """Eq. 2.  W is K x N ([in, out] orientation of the GPT-2 projection
    modules named in Sec. IV-C).  gran: "tensor" (one scale) or "channel"
    (one scale per output channel n, Fig. 2(a)).  literal_div: q = round(w / s)
    with a division per element instead of the product with qmax / amax."""
    qmax = qmax_of(bits)
    W32 = _f32(W16)
    K, N = W32.shape
    if gran == "tensor":
        amax = absmax(W32)
        s, inv = scale(amax, qmax)
        wq = quantize_div(W32, s, "tensor", qmax) if literal_div else quantize(W32, inv, qmax)
        return {"w_q": wq, "s_w": np.array([s], np.float32),
                "inv_w": np.array([inv], np.float32), "amax_w": np.array([amax], np.float32)}
    assert gran == "channel"
    amax = col_absmax(W32)
    s = np.empty(N, np.float32)
    inv = np.empty(N, np.float32)
    for n in range(N):
        s[n], inv[n] = scale(amax[n], qmax)
    wq = quantize_div(W32, s, "col", qmax) if literal_div else quantize_cols(W32, inv, qmax)
    return {"w_q": wq, "s_w": s, "inv_w": inv, "amax_w": amax}


def linear(X16, W16=None, *, threshold=6.0, e=2, r_cap=64, w_gran="tensor",
           x_gran="tensor", bias16=None, rows=None, ia_bits=8, w_bits=8,
           wpack=None, static_idx=None, aux_scale="shared", literal_div=False):
    """The whole MUXQ linear layer, step by step.

    aux_scale: "shared" -- Aux is quantised with Body's scale (Eq. 5 read as an
    identity: its codes are Body's outlier columns), so Eq. 7 is summed on the
    integer accumulators; "own" -- Aux gets the abs-max scale of Eq. 1 on its own
    values (one per matrix, or one per token), and Eq. 7 is recombined after
    dequantisation, in fp32.  Both give the same codes whenever max|Body| sits on an
    outlier channel.
    literal_div: the codes are round(v / s) with one fp32 division per element (Eq. 1-2
    as printed) instead of round(v * (qmax / amax)); measures how much that reading
    matters, nothing else uses it.

    static_idx: optional strictly ascending list of channel indices found offline
    (the Sec. III-C criterion applied to calibration data): these channels are
    decomposed whatever the current magnitudes are, the threshold is not used, and
    a list longer than r_cap keeps its r_cap lowest entries.

    X16: M x K activations (fp16 values).  W16: K x N weights (fp16 values),
    or pass wpack = quantize_weight(...) computed earlier.
    rows: optional list of row indices; the integer products, recombination
    and dequantisation are then evaluated for those rows only (everything
    before the products always sees the whole X, as the scales depend on it).
    Returns a dict of every stage output.
    """
    qx = qmax_of(ia_bits)
    X32 = _f32(X16)
    M, K = X32.shape
    out = {}
    # Sec. III-C: detect outlier channels on the raw activations.
    colmax = col_absmax(X32)
    if static_idx is None:
        idx, r, n_total = select_outliers(colmax, threshold, r_cap)
    else:
        lst = [int(k) for k in static_idx]
        assert all(0 <= k < K for k in lst) and all(a < b for a, b in zip(lst, lst[1:]))
        n_total, r = len(lst), min(len(lst), r_cap)
        idx = np.full(r_cap, -1, np.int32)
        idx[:r] = lst[:r]
    out.update(col_absmax=colmax, outlier_idx=idx, n_used=r, n_total=n_total)
    # Eq. 4-5: Body / Aux.
    body, aux = decompose(X32, idx, r, e)
    # Eq. 1 on Body.  Aux is the same values as Body's outlier columns (Eq. 5)
    # and is quantised with Body's scale so that Eq. 7 can be summed in
    # integers.
    assert aux_scale in ("shared", "own")
    auxc = np.ascontiguousarray(aux)
    if x_gran == "tensor":
        amax = absmax(body)
        s_x, inv_x = scale(amax, qx)
        s_x = np.array([s_x], np.float32)
        inv_x = np.array([inv_x], np.float32)
        if aux_scale == "own" and r:
            amax_aux = absmax(auxc)
            s_a, inv_a = scale(amax_aux, qx)
            s_aux, inv_aux = np.array([s_a], np.float32), np.array([inv_a], np.float32)
        else:
            s_aux, inv_aux = s_x, inv_x
        if literal_div:
            body_q = quantize_div(body, s_x, "tensor", qx)
            aux_q = quantize_div(auxc, s_aux, "tensor", qx) if r else np.zeros((M, 0), np.int8)
        else:
            body_q = quantize(body, inv_x[0], qx)
            aux_q = quantize(auxc, inv_aux[0], qx) if r else np.zeros((M, 0), np.int8)
    else:
        assert x_gran == "token"
        amax = row_absmax(body)
        s_x = np.empty(M, np.float32)
        inv_x = np.empty(M, np.float32)
        for m in range(M):
            s_x[m], inv_x[m] = scale(amax[m], qx)
        if aux_scale == "own" and r:
            amax_aux = row_absmax(auxc)
            s_aux = np.empty(M, np.float32)
            inv_aux = np.empty(M, np.float32)
            for m in range(M):
                s_aux[m], inv_aux[m] = scale(amax_aux[m], qx)
        else:
            s_aux, inv_aux = s_x, inv_x
        if literal_div:
            body_q = quantize_div(body, s_x, "row", qx)
            aux_q = quantize_div(auxc, s_aux, "row", qx) if r else np.zeros((M, 0), np.int8)
        else:
            body_q = quantize_rows(body, inv_x, qx)
            aux_q = quantize_rows(auxc, inv_aux, qx) if r else np.zeros((M, 0), np.int8)
    out.update(body=body, aux=aux, amax_body=amax, s_x=s_x, inv_x=inv_x, s_aux=s_aux,
               inv_aux=inv_aux, body_q=body_q, aux_q=aux_q)
    if W16 is None and wpack is None:
        return out
    # Eq. 2 on W (offline in deployment).
    if wpack is None:
        wpack = quantize_weight(W16, w_gran, w_bits, literal_div=literal_div)
    w_q, s_w = wpack["w_q"], wpack["s_w"]
    out.update(w_q=w_q, s_w=s_w)
    N = w_q.shape[1]
    # Eq. 7 on integer codes.
    if rows is not None:
        rows = np.asarray(rows, np.int64)
        bq, aq = body_q[rows], aux_q[rows]
    else:
        bq, aq = body_q, aux_q
    acc_body = gemm_i8(bq, w_q)
    if r:
        w_rows = gather_rows(w_q, idx, r)
        acc_aux = gemm_i8(aq, w_rows)
    else:
        acc_aux = np.zeros_like(acc_body)
    bias32 = _f32(bias16) if bias16 is not None else None
    sx_used = s_x if (x_gran == "tensor" or rows is None) else s_x[rows]
    if aux_scale == "own":
        # Eq. 7 in real numbers: the two products sit on different scales
        sa_used = s_aux if (x_gran == "tensor" or rows is None) else s_aux[rows]
        out.update(acc_body=acc_body, acc_aux=acc_aux, acc=None, rows=rows)
        y32 = dequant_sum(acc_body, acc_aux, sx_used, sa_used, s_w, e, bias32)
    else:
        acc = recombine(acc_body, acc_aux, e)
        out.update(acc_body=acc_body, acc_aux=acc_aux, acc=acc, rows=rows)
        # Eq. 3.
        y32 = dequant(acc, sx_used, s_w, bias32)
    with np.errstate(over="ignore"):          # beyond 65504 rounds to inf, as fp16 does
        y16 = y32.astype(np.float16)
    out.update(y32=y32, y16=y16)
    return out


# ------------------------------------------- the paper's evaluation route ----

def fake_quant_linear(X16, W16, *, muxq=True, threshold=6.0, e=2, r_cap=64, w_gran="tensor",
                      x_gran="tensor", ia_bits=8, w_bits=8, aux_scale="shared"):
    """Sec. IV-C: the layer as the paper's own experiments evaluate it -- operands are
    quantised and immediately dequantised, and the product is taken in floating
    point (fp64 here).  With muxq=True the activation is decomposed first
    (Eq. 4-5), Body and Aux are quantised and dequantised, and X is rebuilt by
    Eq. 6 before the product; with muxq=False it is the naive quantiser of
    Eq. 1-3.  In exact arithmetic this equals s_x * s_w * (acc_body + (2^e - 1) *
    acc_aux) of the integer route (Eq. 7), which is what the tests hold it to.
    Returns the M x N fp64 result."""
    o = linear(X16, None, threshold=threshold, e=e, r_cap=r_cap if muxq else 0,
               x_gran=x_gran, ia_bits=ia_bits, aux_scale=aux_scale)
    wp = quantize_weight(W16, w_gran, w_bits)
    s_x = o["s_x"].astype(np.float64).reshape(-1, 1)          # [1,1] or [M,1]
    body_hat = s_x * o["body_q"].astype(np.float64)
    x_hat = body_hat
    r = o["n_used"]
    if r:
        aux_hat = o["s_aux"].astype(np.float64).reshape(-1, 1) * o["aux_q"].astype(np.float64)
        cols = o["outlier_idx"][:r]
        x_hat[:, cols] += float((1 << e) - 1) * aux_hat       # Eq. 6
    w_hat = wp["w_q"].astype(np.float64) * wp["s_w"].astype(np.float64).reshape(1, -1)
    return x_hat @ w_hat


def sqnr_db(y, y_ref):
    """10 log10( sum y_ref^2 / sum (y - y_ref)^2 ): the accuracy figure used in place of
    the perplexities of Tables 1-2, which need the dataset and the trained weights."""
    y = np.asarray(y, np.float64)
    y_ref = np.asarray(y_ref, np.float64)
    err = float(((y - y_ref) ** 2).sum())
    sig = float((y_ref ** 2).sum())
    if err == 0.0:
        return float("inf")
    return 10.0 * np.log10(sig / err)


def gelu_tanh(Y16):
    """The GELU of the GPT-2 MLP (between the two projections of Sec. IV-C), tanh form:
    gelu(y) = 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3))), evaluated in fp64 on the
    fp16 input and rounded once to fp16 (round-to-nearest-even)."""
    y = np.asarray(Y16, dtype=np.float16).astype(np.float64)
    u = np.sqrt(2.0 / np.pi) * (y + 0.044715 * y * y * y)
    return (0.5 * y * (1.0 + np.tanh(u))).astype(np.float16)


def mlp(X16, W1_16, b1_16, W2_16, b2_16, **kw):
    """The MLP of a GPT-2 block as the method wraps it (Sec. IV-C): c_fc, the tanh GELU,
    c_proj, with both projections running as MUXQ linear layers (options `kw` go to both).
    Every piece is the plain function above: linear -> gelu_tanh on its fp16 output -> linear.
    Returns (hidden fp16 after the GELU, the second layer's result dict)."""
    h = linear(X16, W1_16, bias16=b1_16, **kw)["y16"]
    g = gelu_tanh(h)
    return g, linear(g, W2_16, bias16=b2_16, **kw)
