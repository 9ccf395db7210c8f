"""Exact-arithmetic brute force of the MUXQ linear layer, for tiny inputs.

Independent of the C oracle and of numpy's float arithmetic: every value is a
Python ``Fraction`` or ``int``; binary32 rounding is done by ``fl32`` below
(round-to-nearest-even on the 24-bit significand, written out by hand), the
integer products are plain Python loops.  Follows Sec. II-A Eq. 1-3 and
Sec. III-C Eq. 4-7 of the paper directly.
"""
from fractions import Fraction


def rne(fr: Fraction) -> int:
    """Round a rational to the nearest integer, ties to even."""
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def fl32(fr: Fraction) -> Fraction:
    """Nearest IEEE binary32 value (ties to even), subnormals included.
    No overflow handling: inputs here stay far below 2^128."""
    if fr == 0:
        return Fraction(0)
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    n = rne(a / quantum)
    res = n * quantum
    return res if fr > 0 else -res


def quant(v: Fraction, inv: Fraction, qmax: int = 127) -> int:
    q = rne(fl32(v * inv))
    return max(-qmax, min(qmax, q))


def quant_div(v: Fraction, s: Fraction, qmax: int = 127) -> int:
    """Eq. 1-2 as printed: round(v / s), the quotient rounded to binary32 first."""
    if s == 0:
        return 0
    q = rne(fl32(v / s))
    return max(-qmax, min(qmax, q))


def scale_pair(amax: Fraction, qmax: int = 127):
    if amax == 0:
        return Fraction(0), Fraction(0)
    return fl32(amax / qmax), fl32(Fraction(qmax) / amax)


def muxq_linear(X, W, T=Fraction(6), e=2, r_cap=64, w_gran="tensor", bias=None,
                qx=127, qw=127, x_gran="tensor", idx_given=None, aux_scale="shared",
                literal_div=False):
    """X: M x K, W: K x N lists of Fractions (fp16-representable).  Returns a
    dict with idx, body, body_q, aux_q, w_q, s_x, s_w, acc, y32 (Fractions).
    x_gran "token": one activation scale per row of Body (the per-vector
    setting of Sec. II-A / Fig. 2(a)); s_x and inv_x are then lists of M.
    aux_scale "own": Aux is quantised with the abs-max scale of its own values (per matrix,
    or per row with x_gran "token") and Eq. 7 is summed after dequantisation:
    y = fl(fl(fl(s_x s_w) acc_body) + fl(c fl(fl(s_aux s_w) acc_aux))) (+ bias).
    literal_div: codes are round(fl(v / s)) instead of round(fl(v * fl(qmax / amax)))."""
    M, K, N = len(X), len(X[0]), len(W[0])
    colmax = [max(abs(X[m][k]) for m in range(M)) for k in range(K)]
    # idx_given: a list fixed offline replaces the magnitude test
    cand = [k for k in range(K) if colmax[k] > T] if idx_given is None else list(idx_given)
    idx = cand[:r_cap]
    shrink = Fraction(1, 2 ** e)
    body = [[X[m][k] * shrink if k in idx else X[m][k] for k in range(K)] for m in range(M)]
    aux = [[body[m][k] for k in idx] for m in range(M)]
    if x_gran == "tensor":
        amax = max(abs(v) for row in body for v in row)
        s_x, inv_x = scale_pair(amax, qx)
        s_rows, inv_rows = [s_x] * M, [inv_x] * M
    else:
        s_rows, inv_rows = [], []
        for m in range(M):
            s, inv = scale_pair(max(abs(v) for v in body[m]), qx)
            s_rows.append(s)
            inv_rows.append(inv)
        s_x, inv_x = s_rows, inv_rows
    if aux_scale == "own" and idx:
        if x_gran == "tensor":
            sa, ia = scale_pair(max(abs(v) for row in aux for v in row), qx)
            sa_rows, ia_rows = [sa] * M, [ia] * M
        else:
            sa_rows, ia_rows = [], []
            for m in range(M):
                sa, ia = scale_pair(max(abs(v) for v in aux[m]), qx)
                sa_rows.append(sa)
                ia_rows.append(ia)
    else:
        sa_rows, ia_rows = s_rows, inv_rows
    if literal_div:
        body_q = [[quant_div(v, s_rows[m], qx) for v in body[m]] for m in range(M)]
        aux_q = [[quant_div(v, sa_rows[m], qx) for v in aux[m]] for m in range(M)]
    else:
        body_q = [[quant(v, inv_rows[m], qx) for v in body[m]] for m in range(M)]
        aux_q = [[quant(v, ia_rows[m], qx) for v in aux[m]] for m in range(M)]
    if w_gran == "tensor":
        wmax = max(abs(v) for row in W for v in row)
        s, inv = scale_pair(wmax, qw)
        s_w, inv_w = [s] * N, [inv] * N
    else:
        s_w, inv_w = [], []
        for n in range(N):
            s, inv = scale_pair(max(abs(W[k][n]) for k in range(K)), qw)
            s_w.append(s)
            inv_w.append(inv)
    if literal_div:
        w_q = [[quant_div(W[k][n], s_w[n], qw) for n in range(N)] for k in range(K)]
    else:
        w_q = [[quant(W[k][n], inv_w[n], qw) for n in range(N)] for k in range(K)]
    c = 2 ** e - 1
    acc = [[0] * N for _ in range(M)]
    acc_body = [[0] * N for _ in range(M)]
    acc_aux = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            a_body = sum(body_q[m][k] * w_q[k][n] for k in range(K))
            a_aux = sum(aux_q[m][j] * w_q[idx[j]][n] for j in range(len(idx)))
            acc_body[m][n], acc_aux[m][n] = a_body, a_aux
            acc[m][n] = a_body + c * a_aux
    y32 = [[None] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            if aux_scale == "own":
                yb = fl32(fl32(s_rows[m] * s_w[n]) * fl32(Fraction(acc_body[m][n])))
                ya = fl32(fl32(sa_rows[m] * s_w[n]) * fl32(Fraction(acc_aux[m][n])))
                v = fl32(yb + fl32(c * ya))
            else:
                sc = fl32(s_rows[m] * s_w[n])
                v = fl32(sc * fl32(Fraction(acc[m][n])))
            if bias is not None:
                v = fl32(v + bias[n])
            y32[m][n] = v
    return dict(colmax=colmax, idx=idx, n_total=len(cand), body=body, aux=aux,
                body_q=body_q, aux_q=aux_q, w_q=w_q, s_x=s_x, inv_x=inv_x,
                s_aux=sa_rows, s_w=s_w, acc=acc, acc_body=acc_body, acc_aux=acc_aux, y32=y32)
