"""CPU oracle for the Jigsaw linear-layer forward pass.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``jigsaw_oracle.c`` (plain C, IEEE double) plus the
layout definitions (which slice of X / W / b / Y a rank owns) written out as
numpy slicing.  Nothing here is shared with, or imported by, the HIP library or
its Python binding; only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.

Partitioning (all matrices row-major; X is M x K, W is N x K, Y is M x N):

* 2-way (Sec. 4.1): X_r = X[:, r-th half of K], W_r = W[:, r-th half of K]
  (rank r holds all N rows of its W column-half and splits them internally into
  W_{r,0}, W_{r,1}); Y_r = Y[:, r-th half of N].
* 4-way (Sec. 4.2): X_r, W_r, Y_r are the 2 x 2 blocks numbered row-major
  (r = 2*row_half + col_half), as in Eq. (3).
* Bias: b_r is the slice of b matching Y_r's columns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jigsaw_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-pthread", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        lib.oracle_linear.argtypes = [f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_linear_rows.argtypes = [f32p, f32p, f32p, i64, i64, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_magnitude.argtypes = [f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_entries.argtypes = [f32p, f32p, f32p, i64, i64p, i64p, i64, f64p, f64p, ctypes.c_int]
        lib.oracle_jigsaw.argtypes = [ctypes.c_int, f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_backward.argtypes = [f32p, f32p, f32p, i64, i64, i64, f64p, f64p, ctypes.c_int, ctypes.c_int]
        lib.oracle_jigsaw_backward.argtypes = [ctypes.c_int, f32p, f32p, f32p, i64, i64, i64, f64p, f64p,
                                               ctypes.c_int]
        lib.oracle_linear_xtw.argtypes = [f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int, ctypes.c_int]
        lib.oracle_jigsaw_xtw.argtypes = [ctypes.c_int, f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_linear_xw.argtypes = [f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int, ctypes.c_int]
        lib.oracle_jigsaw_xw.argtypes = [ctypes.c_int, f32p, f32p, f32p, i64, i64, i64, f64p, ctypes.c_int]
        lib.oracle_gelu.argtypes = [f64p, i64, f64p]
        lib.oracle_round_bf16.argtypes = [f32p, i64, f32p]
        lib.oracle_layernorm.argtypes = [f32p, f32p, f32p, i64, i64, i64, ctypes.c_double, f64p, f64p, ctypes.c_int]
        lib.oracle_mlp.argtypes = [f32p, f32p, f32p, f32p, f32p, i64, i64, i64, ctypes.c_int,
                                   f64p, f64p, f64p, f64p, f64p, ctypes.c_int]
        for fn in (lib.oracle_linear, lib.oracle_linear_rows, lib.oracle_magnitude,
                   lib.oracle_entries, lib.oracle_jigsaw, lib.oracle_backward, lib.oracle_jigsaw_backward,
                   lib.oracle_linear_xtw, lib.oracle_jigsaw_xtw, lib.oracle_linear_xw, lib.oracle_jigsaw_xw,
                   lib.oracle_gelu, lib.oracle_mlp):
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _opt_f32(a):
    if a is None:
        return None, None
    return _f32(a)


def _f64_out(shape):
    a = np.empty(shape, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle: {what} failed with code {rc}")


def host_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def linear(X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    """Y64 = X W^T + b by the definition, in double."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2 and (b is None or b.shape == (N,))
    Y, yp = _f64_out((M, N))
    _check(_load().oracle_linear(xp, wp, bp, M, K, N, yp, nthreads or host_threads()), "linear")
    return Y


def linear_rows(X, W, b, row_begin: int, row_end: int, nthreads: int | None = None) -> np.ndarray:
    """Rows [row_begin, row_end) of Y64 (returned as a (row_end-row_begin) x N array)."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    N = W.shape[0]
    Y, yp = _f64_out((row_end - row_begin, N))
    _check(_load().oracle_linear_rows(xp, wp, bp, M, K, N, row_begin, row_end, yp,
                                      nthreads or host_threads()), "linear_rows")
    return Y


def magnitude(X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    """S = |b| + |X| |W|^T in double: the scale of the floating-point tolerance."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    N = W.shape[0]
    S, sp = _f64_out((M, N))
    _check(_load().oracle_magnitude(xp, wp, bp, M, K, N, sp, nthreads or host_threads()), "magnitude")
    return S


def entries(Xrows, Wrows, ix, jw, bias_per_entry=None, nthreads: int | None = None):
    """(value, magnitude) of entries e: <Xrows[ix[e]], Wrows[jw[e]]> + bias_per_entry[e]."""
    Xr, xp = _f32(Xrows)
    Wr, wp = _f32(Wrows)
    bj, bp = _opt_f32(bias_per_entry)
    K = Xr.shape[1]
    assert Wr.shape[1] == K
    ix = np.ascontiguousarray(ix, dtype=np.int64)
    jw = np.ascontiguousarray(jw, dtype=np.int64)
    n = ix.shape[0]
    assert jw.shape[0] == n
    assert n == 0 or (ix.min() >= 0 and ix.max() < Xr.shape[0] and jw.min() >= 0 and jw.max() < Wr.shape[0])
    out, op = _f64_out((n,))
    mag, mp = _f64_out((n,))
    i64p = ctypes.POINTER(ctypes.c_int64)
    _check(_load().oracle_entries(xp, wp, bp, K, ix.ctypes.data_as(i64p), jw.ctypes.data_as(i64p),
                                  n, op, mp, nthreads or host_threads()), "entries")
    return out, mag


def jigsaw(ways: int, X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    """Y64 obtained by the method's own steps (shard, block products, exchange, add, gather)."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    N = W.shape[0]
    Y, yp = _f64_out((M, N))
    _check(_load().oracle_jigsaw(ways, xp, wp, bp, M, K, N, yp, nthreads or host_threads()), "jigsaw")
    return Y


def backward(X, W, dY, nthreads: int | None = None, absolute: bool = False):
    """(dX64, dW64) = (dY W, dY^T X) by the definition, in double (magnitudes if ``absolute``)."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    G, gp = _f32(dY)
    M, K = X.shape
    N = W.shape[0]
    assert W.shape[1] == K and G.shape == (M, N)
    dX, dxp = _f64_out((M, K))
    dW, dwp = _f64_out((N, K))
    _check(_load().oracle_backward(xp, wp, gp, M, K, N, dxp, dwp, int(absolute),
                                   nthreads or host_threads()), "backward")
    return dX, dW


def backward_magnitude(X, W, dY, nthreads: int | None = None):
    """(|dY| |W|, |dY|^T |X|): the scales of the backward tolerances."""
    return backward(X, W, dY, nthreads, absolute=True)


def bias_backward(dY, absolute: bool = False) -> np.ndarray:
    """db64 = the gradient of the bias of Y = X W^T + 1 b^T for an incoming gradient dY: its column sums
    db[j] = sum_i dY[i][j], in double, rows ascending (sums of absolute values if ``absolute``)."""
    G = np.ascontiguousarray(dY, dtype=np.float32).astype(np.float64)
    if absolute:
        G = np.abs(G)
    out = np.zeros(G.shape[1], dtype=np.float64)
    for i in range(G.shape[0]):
        out += G[i]
    return out


def jigsaw_backward(ways: int, X, W, dY, nthreads: int | None = None):
    """(dX64, dW64) obtained block by block with dX partitioned like X and dW like W."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    G, gp = _f32(dY)
    M, K = X.shape
    N = W.shape[0]
    dX, dxp = _f64_out((M, K))
    dW, dwp = _f64_out((N, K))
    _check(_load().oracle_jigsaw_backward(ways, xp, wp, gp, M, K, N, dxp, dwp,
                                          nthreads or host_threads()), "jigsaw_backward")
    return dX, dW


def linear_xtw(X, W, b=None, nthreads: int | None = None, absolute: bool = False) -> np.ndarray:
    """Y64 = X^T W + b by the definition (X [T x C], W [T x D], Y [C x D]), in double; the
    magnitude |b| + |X|^T |W| if ``absolute``."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    T, C = X.shape
    T2, D = W.shape
    assert T == T2 and (b is None or b.shape == (D,))
    Y, yp = _f64_out((C, D))
    _check(_load().oracle_linear_xtw(xp, wp, bp, T, C, D, yp, int(absolute), nthreads or host_threads()),
           "linear_xtw")
    return Y


def magnitude_xtw(X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    return linear_xtw(X, W, b, nthreads, absolute=True)


def jigsaw_xtw(ways: int, X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    """Y64 = X^T W + b obtained block by block (the decomposition is stated in the C source)."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    T, C = X.shape
    D = W.shape[1]
    assert W.shape[0] == T
    Y, yp = _f64_out((C, D))
    _check(_load().oracle_jigsaw_xtw(ways, xp, wp, bp, T, C, D, yp, nthreads or host_threads()), "jigsaw_xtw")
    return Y


def backward_xtw(X, W, dY, nthreads: int | None = None, absolute: bool = False):
    """(dX64, dW64) of the transposed layer Y = X^T W (X [T x C], W [T x D], dY [C x D]) by the definition:
    dX[t][c] = sum_d W[t][d] dY[c][d]  and  dW[t][d] = sum_c X[t][c] dY[c][d],  in double - each is a product of
    the form A B^T, evaluated by the forward layer's routine (magnitudes if ``absolute``)."""
    G = np.ascontiguousarray(dY, dtype=np.float32)
    f = magnitude if absolute else linear
    return f(W, G, None, nthreads), f(X, np.ascontiguousarray(G.T), None, nthreads)


def linear_xw(X, W, b=None, nthreads: int | None = None, absolute: bool = False) -> np.ndarray:
    """Y64 = X W + b by the definition (X [M x K], W [K x N], Y [M x N]: the permutation of Sec. 5 whose weights are
    stored along the contracted index), in double; the magnitude |b| + |X| |W| if ``absolute``."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    K2, N = W.shape
    assert K == K2 and (b is None or b.shape == (N,))
    Y, yp = _f64_out((M, N))
    _check(_load().oracle_linear_xw(xp, wp, bp, M, K, N, yp, int(absolute), nthreads or host_threads()), "linear_xw")
    return Y


def magnitude_xw(X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    return linear_xw(X, W, b, nthreads, absolute=True)


def jigsaw_xw(ways: int, X, W, b=None, nthreads: int | None = None) -> np.ndarray:
    """Y64 = X W + b obtained block by block (the decomposition is stated in the C source)."""
    X, xp = _f32(X)
    W, wp = _f32(W)
    b, bp = _opt_f32(b)
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K
    Y, yp = _f64_out((M, N))
    _check(_load().oracle_jigsaw_xw(ways, xp, wp, bp, M, K, N, yp, nthreads or host_threads()), "jigsaw_xw")
    return Y


def backward_xw(X, W, dY, nthreads: int | None = None, absolute: bool = False):
    """(dX64, dW64) of the layer Y = X W (X [M x K], W [K x N], dY [M x N]) by the definition:
    dX[i][k] = sum_j dY[i][j] W[k][j]  (the form A B^T: the forward layer's routine)  and
    dW[k][j] = sum_i X[i][k] dY[i][j]  (the form A^T B: the transposed layer's routine), in double
    (magnitudes if ``absolute``)."""
    G = np.ascontiguousarray(dY, dtype=np.float32)
    f = magnitude if absolute else linear
    return f(G, W, None, nthreads), linear_xtw(X, G, None, nthreads, absolute)


def gelu(a) -> np.ndarray:
    """x * Phi(x), element by element, in double."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty_like(a)
    _check(_load().oracle_gelu(a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), a.size,
                               out.ctypes.data_as(ctypes.POINTER(ctypes.c_double))), "gelu")
    return out


def gelu_grad(a) -> np.ndarray:
    """d/dx (x Phi(x)) = Phi(x) + x phi(x), element by element, in double (Phi, phi: the standard normal
    distribution function and density; erf from the library)."""
    from scipy.special import erf
    a = np.ascontiguousarray(a, dtype=np.float64)
    return 0.5 * (1.0 + erf(a * 0.70710678118654752440)) + a * np.exp(-0.5 * a * a) * 0.39894228040143267794


def mlp_backward(X, W1, b1, W2, dY, nthreads: int | None = None):
    """Gradients of the mixing MLP Y = X + gelu(X W1^T + b1) W2^T + b2 for an incoming gradient dY, in double, by the
    chain rule through the layers' own backward passes (Sec. 4.1), with what the method stores between the steps
    handed on in FP32 (H, dA):
        A = X W1^T + b1,  H = gelu(A);   dH = dY W2,  dW2 = dY^T H,  db2 = sum_i dY;
        dA = dH * gelu'(A);              dX = dY + dA W1,  dW1 = dA^T X,  db1 = sum_i dA.
    Returns a dict with A, dH, dA, dX, dW1, db1, dW2, db2."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    A = linear(X, W1, b1, nthreads)
    H32 = gelu(A).astype(np.float32)
    dH, dW2 = backward(H32, W2, dY, nthreads)
    dA = dH * gelu_grad(A)
    dA32 = dA.astype(np.float32)
    dXm, dW1 = backward(X, W1, dA32, nthreads)
    return dict(A=A, dH=dH, dA=dA, dX=dXm + np.asarray(dY, dtype=np.float64), dW1=dW1, db1=bias_backward(dA32),
                dW2=dW2, db2=bias_backward(dY))


def mlp(X, W1, b1, W2, b2, residual: bool = True, nthreads: int | None = None):
    """One mixing MLP: H = gelu(X W1^T + b1), Y = (X +) H W2^T + b2, in double.

    Returns a dict with H, Y and the magnitudes S1 (pre-activation), SY (second layer's own sums) and
    PY = S1 |W2|^T (how an S1-relative error in H carries into Y)."""
    X, xp = _f32(X)
    W1, w1p = _f32(W1)
    b1, b1p = _opt_f32(b1)
    W2, w2p = _f32(W2)
    b2, b2p = _opt_f32(b2)
    M, C = X.shape
    Hd = W1.shape[0]
    assert W1.shape == (Hd, C) and W2.shape == (C, Hd)
    H, hp = _f64_out((M, Hd))
    Y, yp = _f64_out((M, C))
    S1, s1p = _f64_out((M, Hd))
    SY, syp = _f64_out((M, C))
    PY, pyp = _f64_out((M, C))
    _check(_load().oracle_mlp(xp, w1p, b1p, w2p, b2p, M, C, Hd, int(residual), hp, yp, s1p, syp, pyp,
                              nthreads or host_threads()), "mlp")
    return dict(H=H, Y=Y, S1=S1, SY=SY, PY=PY)


def jigsaw_mlp(ways: int, X, W1, b1, W2, b2, residual: bool = True):
    """The same MLP with both layers obtained block by block (jigsaw), H handed on in FP32 as the
    method stores it, the residual added to the gathered result."""
    H = gelu(jigsaw(ways, X, W1, b1)).astype(np.float32)
    Y = jigsaw(ways, H, W2, b2)
    return Y + np.asarray(X, dtype=np.float64) if residual else Y


# ----------------------------------------------------------------------------
# reduced precision (Sec. 6.1: matrix units that round FP32 operands to a short mantissa, FP32 sums)
# ----------------------------------------------------------------------------
def round_bf16(a) -> np.ndarray:
    """FP32 values rounded to bfloat16 (nearest, ties to even), returned as FP32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    _check(_load().oracle_round_bf16(a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), a.size,
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))), "round_bf16")
    return out


def split_bf16(a):
    """x = hi + lo + (a remainder below 2^-17 |x|): hi = round_bf16(x), lo = round_bf16(x - hi)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    hi = round_bf16(a)
    lo = round_bf16(a - hi)          # the difference is exact in FP32 (pinned)
    return hi, lo


def linear_reduced(X, W, b=None, terms: int = 1, nthreads: int | None = None, absolute: bool = False) -> np.ndarray:
    """The layer Y = X W^T + b with operands rounded to bfloat16, in double.

    terms = 1: round(X) round(W)^T.  terms = 3: split operands, Xhi Whi^T + Xhi Wlo^T + Xlo Whi^T (the
    lo * lo product is dropped).  absolute=True: the same sums of absolute values (the magnitude)."""
    f = magnitude if absolute else linear
    if terms == 1:
        return f(round_bf16(X), round_bf16(W), b, nthreads)
    if terms != 3:
        raise RuntimeError(f"terms must be 1 or 3, not {terms}")
    Xh, Xl = split_bf16(X)
    Wh, Wl = split_bf16(W)
    return f(Xh, Wh, b, nthreads) + f(Xh, Wl, None, nthreads) + f(Xl, Wh, None, nthreads)


def backward_reduced(X, W, dY, terms: int = 1, nthreads: int | None = None, absolute: bool = False):
    """(dX64, dW64) = (dY W, dY^T X) of the layer Y = X W^T in the reduced-precision modes of linear_reduced: every
    operand of a product (dY, W, X) is rounded to bfloat16 (or split) element by element, the products are exact and
    summed in double.  Each gradient is a product of the form A B^T, so it is linear_reduced on transposed operands."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    G = np.ascontiguousarray(dY, dtype=np.float32)
    t = lambda a: np.ascontiguousarray(a.T)
    dX = linear_reduced(G, t(W), None, terms, nthreads, absolute)          # [M x N] [K x N]^T
    dW = linear_reduced(t(G), t(X), None, terms, nthreads, absolute)       # [N x M] [K x M]^T
    return dX, dW


def backward_xtw_reduced(X, W, dY, terms: int = 1, nthreads: int | None = None, absolute: bool = False):
    """(dX64, dW64) = (W dY^T, X dY) of the transposed layer Y = X^T W in the reduced-precision modes: every operand of
    a product rounded (or split) element by element, exact products, double sums - linear_reduced on the operands laid
    out as A B^T."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    G = np.ascontiguousarray(dY, dtype=np.float32)
    dX = linear_reduced(W, G, None, terms, nthreads, absolute)                                # [T x D] [C x D]^T
    dW = linear_reduced(X, np.ascontiguousarray(G.T), None, terms, nthreads, absolute)       # [T x C] [D x C]^T
    return dX, dW


def linear_xtw_reduced(X, W, b=None, terms: int = 1, nthreads: int | None = None, absolute: bool = False) -> np.ndarray:
    """The transposed layer Y = X^T W + b (X [T x C], W [T x D]) in the reduced-precision modes of linear_reduced:
    the rounding (or the split) acts element by element, so it is that function on the transposed operands."""
    Xt = np.ascontiguousarray(np.asarray(X, dtype=np.float32).T)
    Wt = np.ascontiguousarray(np.asarray(W, dtype=np.float32).T)
    return linear_reduced(Xt, Wt, b, terms, nthreads, absolute)


def mlp_reduced(X, W1, b1, W2, b2, terms: int = 1, residual: bool = True, nthreads: int | None = None):
    """One mixing MLP in the mixed precision of Sec. 6.1: both matrix products take their operands rounded to
    bfloat16 (split in two for terms = 3) and sum exactly; bias, GELU and the skip connection are not rounded; H
    is stored in FP32 between the layers, as the method stores every activation, and is rounded like any other
    operand when the second product reads it.  Returns H, Y (double) and the magnitudes S1 (pre-activation) and
    SY (the second layer's own sums, from the stored H)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    S1 = linear_reduced(X, W1, b1, terms, nthreads, absolute=True)
    H = gelu(linear_reduced(X, W1, b1, terms, nthreads))
    H32 = H.astype(np.float32)
    Y = linear_reduced(H32, W2, b2, terms, nthreads)
    SY = linear_reduced(H32, W2, b2, terms, nthreads, absolute=True)
    if residual:
        Y = Y + X.astype(np.float64)
        SY = SY + np.abs(X.astype(np.float64))
    return dict(H=H, Y=Y, S1=S1, SY=SY)


# ----------------------------------------------------------------------------
# layer norm (Sec. 3; Sec. 5 "Layer norms") and the pre-norm channel-mixing block
# ----------------------------------------------------------------------------
LN_EPS = 1e-5      # the default of the library routine the paper says it uses


def ln_groups(ways: int) -> int:
    """Channel blocks that are normalised on their own: the channels are split in two for 2- and 4-way."""
    if ways not in (1, 2, 4):
        raise RuntimeError(f"ways must be 1, 2 or 4, not {ways}")
    return 1 if ways == 1 else 2


def layernorm(X, gamma=None, beta=None, groups: int = 1, eps: float = LN_EPS, nthreads: int | None = None,
              magnitude: bool = False):
    """Per token (row) and channel block: (x - mean) / sqrt(var + eps) * gamma + beta, in double.

    With magnitude=True also returns (|x| + |mean|) / sqrt(var + eps) * |gamma| + |beta|."""
    X, xp = _f32(X)
    gamma, gp = _opt_f32(gamma)
    beta, bp = _opt_f32(beta)
    M, C = X.shape
    assert gamma is None or gamma.shape == (C,)
    assert beta is None or beta.shape == (C,)
    Y, yp = _f64_out((M, C))
    S, sp = _f64_out((M, C)) if magnitude else (None, None)
    _check(_load().oracle_layernorm(xp, gp, bp, M, C, groups, float(eps), yp, sp, nthreads or host_threads()),
           "layernorm")
    return (Y, S) if magnitude else Y


def layernorm_backward(X, gamma, dY, groups: int = 1, eps: float = LN_EPS, magnitude: bool = False):
    """Gradients of Y = layernorm(X, gamma, beta, groups, eps) for an incoming gradient dY, in double.  Per token and
    channel block of n channels, with xhat = (x - mean) / sqrt(var + eps) and g = dY * gamma:
        dX     = (g - mean_c(g) - xhat * mean_c(g * xhat)) / sqrt(var + eps)
        dgamma = sum over tokens of dY * xhat,     dbeta = sum over tokens of dY
    (the derivative of the definition: mean and variance depend on every channel of the block).  Returns
    (dX, dgamma, dbeta); with magnitude=True also the sums of absolute values of the terms of each
    (SX = (|g| + mean|g| + |xhat| mean|g xhat|) rstd, Sg = sum |dY xhat|, Sb = sum |dY|)."""
    X = np.ascontiguousarray(X, dtype=np.float32).astype(np.float64)
    G = np.ascontiguousarray(dY, dtype=np.float32).astype(np.float64)
    M, C = X.shape
    if groups < 1 or C % groups:
        raise RuntimeError(f"{C} channels do not split into {groups} blocks")
    if not eps >= 0:
        raise RuntimeError("eps must be >= 0")
    ga = np.ones(C) if gamma is None else np.ascontiguousarray(gamma, dtype=np.float32).astype(np.float64)
    n = C // groups
    dX = np.empty((M, C)); SX = np.empty((M, C))
    xhat = np.empty((M, C))
    for b in range(groups):
        sl = slice(b * n, (b + 1) * n)
        x = X[:, sl]
        mu = x.mean(axis=1, keepdims=True)
        rstd = 1.0 / np.sqrt(((x - mu) ** 2).mean(axis=1, keepdims=True) + eps)
        xh = (x - mu) * rstd
        g = G[:, sl] * ga[sl]
        dX[:, sl] = (g - g.mean(axis=1, keepdims=True) - xh * (g * xh).mean(axis=1, keepdims=True)) * rstd
        SX[:, sl] = (np.abs(g) + np.abs(g).mean(axis=1, keepdims=True)
                     + np.abs(xh) * np.abs(g * xh).mean(axis=1, keepdims=True)) * rstd
        xhat[:, sl] = xh
    dgamma, dbeta = (G * xhat).sum(axis=0), G.sum(axis=0)
    if magnitude:
        return dX, dgamma, dbeta, SX, np.abs(G * xhat).sum(axis=0), np.abs(G).sum(axis=0)
    return dX, dgamma, dbeta


def mixing_block(ways: int, X, gamma, beta, W1, b1, W2, b2, eps: float = LN_EPS):
    """Channel-mixing half of a mixing block (Sec. 3: layer norm before the MLP, skip connection around it):
    Xn = layernorm(X), H = gelu(Xn W1^T + b1), Y = X + H W2^T + b2, with Xn handed on in FP32 as the
    method stores it.  Returns a dict like mlp() plus Xn (double, before rounding)."""
    Xn = layernorm(X, gamma, beta, ln_groups(ways), eps)
    out = mlp(Xn.astype(np.float32), W1, b1, W2, b2, residual=False)
    out["Y"] = out["Y"] + np.asarray(X, dtype=np.float64)
    out["SY"] = out["SY"] + np.abs(np.asarray(X, dtype=np.float64))
    out["Xn"] = Xn
    return out


def mixing_block_backward(ways: int, X, gamma, beta, W1, b1, W2, dY, eps: float = LN_EPS):
    """Gradients of mixing_block (Y = X + MLP(layernorm(X))) for an incoming gradient dY, in double: the MLP's
    backward on Xn without its skip connection, then the norm's backward, then the block's own skip connection;
    Xn and dXn handed on in FP32.  Returns the dict of mlp_backward (its dX is replaced by the block's) plus dXn,
    dgamma, dbeta."""
    G = np.asarray(dY, dtype=np.float64)
    Xn32 = layernorm(X, gamma, beta, ln_groups(ways), eps).astype(np.float32)
    r = mlp_backward(Xn32, W1, b1, W2, dY)
    dXn = r["dX"] - G                               # the MLP's share: dA W1
    dXl, dgamma, dbeta = layernorm_backward(X, gamma, dXn.astype(np.float32), ln_groups(ways), eps)
    r.update(dXn=dXn, dX=G + dXl, dgamma=dgamma, dbeta=dbeta)
    return r


def mlp_backward_reduced(X, W1, b1, W2, dY, terms: int = 1, nthreads: int | None = None):
    """mlp_backward with every product in mixed precision (linear_reduced, backward_reduced): the operands of each
    product are rounded (or split) from the FP32 values the method keeps; A, H, dH, dA, the GELU derivative, the
    bias gradients and the skip connection stay in full precision."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    A = linear_reduced(X, W1, b1, terms, nthreads)
    H32 = gelu(A).astype(np.float32)
    dH, dW2 = backward_reduced(H32, W2, dY, terms, nthreads)
    dA = dH * gelu_grad(A)
    dA32 = dA.astype(np.float32)
    dXm, dW1 = backward_reduced(X, W1, dA32, terms, nthreads)
    return dict(A=A, dH=dH, dA=dA, dX=dXm + np.asarray(dY, dtype=np.float64), dW1=dW1, db1=bias_backward(dA32),
                dW2=dW2, db2=bias_backward(dY))


def mixing_block_backward_reduced(ways: int, X, gamma, beta, W1, b1, W2, dY, terms: int = 1, eps: float = LN_EPS):
    """mixing_block_backward with the MLP's products in mixed precision (mlp_backward_reduced); the norm in full."""
    G = np.asarray(dY, dtype=np.float64)
    Xn32 = layernorm(X, gamma, beta, ln_groups(ways), eps).astype(np.float32)
    r = mlp_backward_reduced(Xn32, W1, b1, W2, dY, terms)
    dXn = r["dX"] - G
    dXl, dgamma, dbeta = layernorm_backward(X, gamma, dXn.astype(np.float32), ln_groups(ways), eps)
    r.update(dXn=dXn, dX=G + dXl, dgamma=dgamma, dbeta=dbeta)
    return r


def mixing_block_reduced(ways: int, X, gamma, beta, W1, b1, W2, b2, terms: int = 1, eps: float = LN_EPS):
    """mixing_block with the MLP's two products in mixed precision (mlp_reduced); the layer norm, its FP32
    output Xn and the skip connection stay in full precision."""
    Xn = layernorm(X, gamma, beta, ln_groups(ways), eps)
    out = mlp_reduced(Xn.astype(np.float32), W1, b1, W2, b2, terms, residual=False)
    out["Y"] = out["Y"] + np.asarray(X, dtype=np.float64)
    out["SY"] = out["SY"] + np.abs(np.asarray(X, dtype=np.float64))
    out["Xn"] = Xn
    return out


def token_mixing_block(ways: int, X, gamma, beta, W1, b1, W2, b2, eps: float = LN_EPS):
    """Token-mixing half of a mixing block (Sec. 3: the MLP applied along the token dimension of the layer-normed
    input, skip connection around it).  X is [T x C]; every channel's column of T token values goes through
        y_c = x_c + W2 gelu(W1^T xn_c + b1) + b2,     W1, W2: [T x D], b1: [D], b2: [T],
    with xn the layer norm of X over each token's channels (as in the channel-mixing half).  In matrix form, with
    the steps taken in the layouts the layers use: H = gelu(Xn^T W1 + b1) is [C x D] (the transposed layer of Sec. 5),
    and Y = X + W2 H^T + b2 1^T is [T x C] again - a plain X W^T layer with W2 in the activations' place and H in the
    weights' place, so nothing is ever transposed.  Xn and H are handed on in FP32 as the method stores them.
    Returns H, Y, Xn (double) and the magnitudes S1 (pre-activation) and SY (the second layer's own sums plus |X|, |b2|)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    Xn = layernorm(X, gamma, beta, ln_groups(ways), eps)
    Xn32 = Xn.astype(np.float32)
    S1 = linear_xtw(Xn32, W1, b1, absolute=True)
    H = gelu(linear_xtw(Xn32, W1, b1))
    H32 = H.astype(np.float32)
    b2 = np.asarray(b2, dtype=np.float64)
    Y = X.astype(np.float64) + linear(W2, H32) + b2[:, None]
    SY = np.abs(X.astype(np.float64)) + magnitude(W2, H32) + np.abs(b2)[:, None]
    return dict(H=H, Y=Y, Xn=Xn, S1=S1, SY=SY)


def token_mixing_block_reduced(ways: int, X, gamma, beta, W1, b1, W2, b2, terms: int = 1, eps: float = LN_EPS):
    """token_mixing_block with its two products in mixed precision (linear_xtw_reduced, linear_reduced): the operands
    of each product are rounded (or split), the layer norm, Xn, H, the skip connection and both biases stay FP32.
    Returns H, Y, Xn (double) and the magnitudes S1, SY of the rounded operands' products."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    Xn = layernorm(X, gamma, beta, ln_groups(ways), eps)
    Xn32 = Xn.astype(np.float32)
    S1 = linear_xtw_reduced(Xn32, W1, b1, terms, absolute=True)
    H = gelu(linear_xtw_reduced(Xn32, W1, b1, terms))
    H32 = H.astype(np.float32)
    b2 = np.asarray(b2, dtype=np.float64)
    Y = X.astype(np.float64) + linear_reduced(W2, H32, None, terms) + b2[:, None]
    SY = np.abs(X.astype(np.float64)) + linear_reduced(W2, H32, None, terms, absolute=True) + np.abs(b2)[:, None]
    return dict(H=H, Y=Y, Xn=Xn, S1=S1, SY=SY)


def token_mixing_block_backward_reduced(ways: int, X, gamma, beta, W1, b1, W2, dY, terms: int = 1, eps: float = LN_EPS):
    """token_mixing_block_backward with every product in mixed precision (linear_xtw_reduced, backward_reduced,
    backward_xtw_reduced); the norm, the GELU derivative, the bias gradients and the skip connection in full."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    G32 = np.ascontiguousarray(dY, dtype=np.float32)
    Xn32 = layernorm(X, gamma, beta, ln_groups(ways), eps).astype(np.float32)
    A = linear_xtw_reduced(Xn32, W1, b1, terms)
    H32 = gelu(A).astype(np.float32)
    dW2, dH = backward_reduced(W2, H32, G32, terms)
    dA = dH * gelu_grad(A)
    dA32 = dA.astype(np.float32)
    dXn, dW1 = backward_xtw_reduced(Xn32, W1, dA32, terms)
    dXl, dgamma, dbeta = layernorm_backward(X, gamma, dXn.astype(np.float32), ln_groups(ways), eps)
    return dict(A=A, dH=dH, dA=dA, dXn=dXn, dX=G32.astype(np.float64) + dXl, dW1=dW1, db1=bias_backward(dA32),
                dW2=dW2, db2=bias_backward(np.ascontiguousarray(G32.T)), dgamma=dgamma, dbeta=dbeta)


def token_mixing_block_backward(ways: int, X, gamma, beta, W1, b1, W2, dY, eps: float = LN_EPS):
    """Gradients of token_mixing_block for an incoming gradient dY [T x C], in double, by the chain rule through the
    steps in the layouts the layers use, with what the method stores between the steps handed on in FP32:
        Xn = layernorm(X),  A = Xn^T W1 + b1 [C x D],  H = gelu(A);
        second layer (W2 in the activations' place, H in the weights'):  dW2 = dY H,  dH = dY^T W2,
        db2[t] = sum_c dY[t][c];   dA = dH * gelu'(A);
        transposed layer:  dXn = W1 dA^T,  dW1 = Xn dA,  db1 = sum_c dA;
        dX = dY + layernorm'(dXn),  dgamma, dbeta from the norm.
    Returns a dict with A, dH, dA, dXn, dX, dW1, db1, dW2, db2, dgamma, dbeta."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    G32 = np.ascontiguousarray(dY, dtype=np.float32)
    Xn32 = layernorm(X, gamma, beta, ln_groups(ways), eps).astype(np.float32)
    A = linear_xtw(Xn32, W1, b1)
    H32 = gelu(A).astype(np.float32)
    dW2, dH = backward(W2, H32, G32)
    db2 = bias_backward(np.ascontiguousarray(G32.T))
    dA = dH * gelu_grad(A)
    dA32 = dA.astype(np.float32)
    dXn, dW1 = backward_xtw(Xn32, W1, dA32)
    dXl, dgamma, dbeta = layernorm_backward(X, gamma, dXn.astype(np.float32), ln_groups(ways), eps)
    return dict(A=A, dH=dH, dA=dA, dXn=dXn, dX=G32.astype(np.float64) + dXl, dW1=dW1, db1=bias_backward(dA32),
                dW2=dW2, db2=db2, dgamma=dgamma, dbeta=dbeta)


# ----------------------------------------------------------------------------
# patch encoder / decoder (Sec. 5 "Encoding and decoding layers"): a convolution whose kernel
# equals its stride is a linear layer over non-overlapping patches
# ----------------------------------------------------------------------------
def patchify(field: np.ndarray, p: int) -> np.ndarray:
    """Patch matrix of a [C, H, W] field: row t = py * (W / p) + px is the patch at (py, px), column
    f = c * p * p + dy * p + dx holds field[c, py * p + dy, px * p + dx].  Plain loops over patches."""
    C, H, W = field.shape
    if p < 1 or H % p or W % p:
        raise ValueError("H and W must be multiples of the patch size")
    hp, wp = H // p, W // p
    out = np.empty((hp * wp, C * p * p), dtype=field.dtype)
    for py in range(hp):
        for px in range(wp):
            for c in range(C):
                blk = field[c, py * p:(py + 1) * p, px * p:(px + 1) * p]
                out[py * wp + px, c * p * p:(c + 1) * p * p] = blk.reshape(-1)
    return out


def unpatchify(patches: np.ndarray, C: int, H: int, W: int, p: int) -> np.ndarray:
    """Inverse of :func:`patchify` (the decoder's rearrangement of token rows back into a field)."""
    hp, wp = H // p, W // p
    assert patches.shape == (hp * wp, C * p * p)
    field = np.empty((C, H, W), dtype=patches.dtype)
    for py in range(hp):
        for px in range(wp):
            for c in range(C):
                field[c, py * p:(py + 1) * p, px * p:(px + 1) * p] = \
                    patches[py * wp + px, c * p * p:(c + 1) * p * p].reshape(p, p)
    return field


def patch_conv(field: np.ndarray, kernel: np.ndarray, bias=None) -> np.ndarray:
    """The encoder by its definition as a strided convolution, in double:
    out[(py, px), n] = b[n] + sum_{c, dy, dx} field[c, py p + dy, px p + dx] * kernel[n, c, dy, dx].
    Pure-Python loops: tiny shapes only."""
    C, H, W = field.shape
    N, C2, p, p2 = kernel.shape
    assert C2 == C and p2 == p and H % p == 0 and W % p == 0
    hp, wp = H // p, W // p
    out = np.zeros((hp * wp, N))
    for py in range(hp):
        for px in range(wp):
            for n in range(N):
                acc = float(bias[n]) if bias is not None else 0.0
                for c in range(C):
                    for dy in range(p):
                        for dx in range(p):
                            acc += float(field[c, py * p + dy, px * p + dx]) * float(kernel[n, c, dy, dx])
                out[py * wp + px, n] = acc
    return out


# ----------------------------------------------------------------------------
# layout definitions (pure indexing; bit-exact)
# ----------------------------------------------------------------------------
def _check_ways(ways, M, K, N):
    if ways not in (1, 2, 4):
        raise ValueError("ways must be 1, 2 or 4")
    if ways >= 2 and (K % 2 or N % 2):
        raise ValueError("K and N must be even")
    if ways == 4 and M % 2:
        raise ValueError("M must be even")


def shard_x(X: np.ndarray, ways: int):
    M, K = X.shape
    _check_ways(ways, M, K, 0)
    if ways == 1:
        return [np.ascontiguousarray(X)]
    if ways == 2:
        return [np.ascontiguousarray(X[:, r * (K // 2):(r + 1) * (K // 2)]) for r in range(2)]
    return [np.ascontiguousarray(X[(r // 2) * (M // 2):(r // 2 + 1) * (M // 2),
                                   (r % 2) * (K // 2):(r % 2 + 1) * (K // 2)]) for r in range(4)]


def shard_w(W: np.ndarray, ways: int):
    N, K = W.shape
    _check_ways(ways, 0, K, N)
    if ways == 1:
        return [np.ascontiguousarray(W)]
    if ways == 2:
        return [np.ascontiguousarray(W[:, r * (K // 2):(r + 1) * (K // 2)]) for r in range(2)]
    return [np.ascontiguousarray(W[(r // 2) * (N // 2):(r // 2 + 1) * (N // 2),
                                   (r % 2) * (K // 2):(r % 2 + 1) * (K // 2)]) for r in range(4)]


def shard_blocks(A: np.ndarray, ways: int):
    """The partition every matrix of the method uses: whole (1-way), column halves (2-way),
    2 x 2 blocks with block (i, j) at position 2 i + j (4-way)."""
    R, Cc = A.shape
    if ways not in (1, 2, 4):
        raise ValueError("ways must be 1, 2 or 4")
    if ways >= 2 and Cc % 2:
        raise ValueError("the number of columns must be even")
    if ways == 4 and R % 2:
        raise ValueError("the number of rows must be even")
    if ways == 1:
        return [np.ascontiguousarray(A)]
    if ways == 2:
        return [np.ascontiguousarray(A[:, r * (Cc // 2):(r + 1) * (Cc // 2)]) for r in range(2)]
    return [np.ascontiguousarray(A[(r // 2) * (R // 2):(r // 2 + 1) * (R // 2),
                                   (r % 2) * (Cc // 2):(r % 2 + 1) * (Cc // 2)]) for r in range(4)]


def shard_b(b: np.ndarray, ways: int):
    (N,) = b.shape
    _check_ways(ways, 0, 0, N)
    if ways == 1:
        return [np.ascontiguousarray(b)]
    if ways == 2:
        return [np.ascontiguousarray(b[r * (N // 2):(r + 1) * (N // 2)]) for r in range(2)]
    return [np.ascontiguousarray(b[(r % 2) * (N // 2):(r % 2 + 1) * (N // 2)]) for r in range(4)]


def shard_y(Y: np.ndarray, ways: int):
    """Y is partitioned like X: column halves (2-way) or 2 x 2 blocks (4-way)."""
    M, N = Y.shape
    _check_ways(ways, M, 0, N)
    if ways == 1:
        return [np.ascontiguousarray(Y)]
    if ways == 2:
        return [np.ascontiguousarray(Y[:, r * (N // 2):(r + 1) * (N // 2)]) for r in range(2)]
    return [np.ascontiguousarray(Y[(r // 2) * (M // 2):(r // 2 + 1) * (M // 2),
                                   (r % 2) * (N // 2):(r % 2 + 1) * (N // 2)]) for r in range(4)]


def gather_y(shards, ways: int) -> np.ndarray:
    if ways == 1:
        return np.ascontiguousarray(shards[0])
    if ways == 2:
        return np.concatenate(shards, axis=1)
    return np.concatenate([np.concatenate(shards[0:2], axis=1),
                           np.concatenate(shards[2:4], axis=1)], axis=0)


# ----------------------------------------------------------------------------
# Freivalds' check: the exact product applied to a vector, at O(MK + NK) cost
# ----------------------------------------------------------------------------
def freivalds_reference(X, W, b, v, chunk_rows: int = 4096):
    """(Y64 @ v, bound) without forming Y: X (W^T v) + <b, v> in double.

    ``v`` is a length-N vector or an N x nv matrix of vectors (one pass over X serves all
    of them).  ``bound = S @ |v|`` is the scale of the tolerance for each projected row.
    """
    W64 = np.asarray(W, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    single = v.ndim == 1
    V = v.reshape(v.shape[0], -1)
    U = W64.T @ V
    Ua = np.abs(W64).T @ np.abs(V)
    if b is None:
        bv = ba = np.zeros(V.shape[1])
    else:
        b64 = np.asarray(b, dtype=np.float64)
        bv, ba = b64 @ V, np.abs(b64) @ np.abs(V)
    M = X.shape[0]
    yv = np.empty((M, V.shape[1]), dtype=np.float64)
    bound = np.empty((M, V.shape[1]), dtype=np.float64)
    for r0 in range(0, M, chunk_rows):
        xc = np.asarray(X[r0:r0 + chunk_rows], dtype=np.float64)
        yv[r0:r0 + chunk_rows] = xc @ U + bv
        bound[r0:r0 + chunk_rows] = np.abs(xc) @ Ua + ba
    if single:
        return yv[:, 0], bound[:, 0]
    return yv, bound


def freivalds_backward(X, W, dY, v, chunk_rows: int = 4096):
    """Projections of the gradients on vectors ``v`` (K x nv): dX v = dY (W v), dW v = dY^T (X v).

    Returns ``(dXv, bound_dX, dWv, bound_dW)``; the bounds are the magnitudes projected on |v|.
    """
    V = np.asarray(v, dtype=np.float64)
    V = V.reshape(V.shape[0], -1)
    W64 = np.asarray(W, dtype=np.float64)
    Wv, Wa = W64 @ V, np.abs(W64) @ np.abs(V)                  # N x nv
    M, N = dY.shape
    dXv = np.empty((M, V.shape[1])); bX = np.empty((M, V.shape[1]))
    dWv = np.zeros((N, V.shape[1])); bW = np.zeros((N, V.shape[1]))
    for r0 in range(0, M, chunk_rows):
        g = np.asarray(dY[r0:r0 + chunk_rows], dtype=np.float64)
        x = np.asarray(X[r0:r0 + chunk_rows], dtype=np.float64)
        dXv[r0:r0 + chunk_rows] = g @ Wv
        bX[r0:r0 + chunk_rows] = np.abs(g) @ Wa
        dWv += g.T @ (x @ V)
        bW += np.abs(g).T @ (np.abs(x) @ np.abs(V))
    return dXv, bX, dWv, bW
