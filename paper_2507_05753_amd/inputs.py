"""Seeded synthetic inputs for the Jigsaw linear layer (X, W, b).

This module only draws numbers.  It holds none of the method's arithmetic (no
products, no sums over k, no block logic) and is the one piece of code that
both the CPU oracle's tests and the HIP path's tests / benchmark may share.

Key stream.  ``key(seed, i)`` is the i-th output (i = 0, 1, ...) of the public
splitmix64 generator started at state ``seed``: the state advances by the
64-bit golden-ratio constant and is passed through the splitmix64 finaliser.
The finaliser is a bijection of the counter, so the keys of one stream are
distinct, and the stream is counter-based, so any sub-range (a row, a sampled
entry) can be produced on its own, on the host (numpy) or on a device (torch
integer ops), with identical bits.

Value maps (all results are exactly representable in FP32):

* mode ``"R"``: the top 24 bits of the key, centred, times 2**-23: uniform on
  a grid in [-1, 1).  Stands in for Z-score-normalised atmospheric fields
  (zero mean, bounded) that the paper's model consumes (Sec. 6, data
  normalisation).
* mode ``"L"``: the top 4 bits of the key, centred, times 2**-3: multiples of
  1/8 in [-1, 0.875].  With power-of-two scaling every partial sum of a dot
  product of such values is exact in FP32 for any summation order, which makes
  bit-exact comparison of a GEMM possible.
* mode ``"Z"`` (host only): a Zipf(s)-distributed rank over a 2**32 domain,
  drawn by inverting the continuous approximation of the Zipf CDF in float64,
  is hashed with the same finaliser and mapped like mode R.  Duplicates are
  kept: the layer has no distinctness requirement on its inputs.

Matrix element (r, c) of a ``rows x cols`` matrix uses counter ``r*cols + c``.
Streams: X uses ``seed``, W uses ``seed + 1000`` (scaled by 2**-6, a power of
two close to 1/sqrt(K) for the paper's channel counts), b uses ``seed + 2000``.
"""
from __future__ import annotations

import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1

W_STREAM = 1000
B_STREAM = 2000
W_SCALE_EXP = -6

ZIPF_S = 1.1
ZIPF_DOMAIN = float(2 ** 32)


# ----------------------------------------------------------------------------
# host (numpy)
# ----------------------------------------------------------------------------
def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (returns a new array)."""
    z = np.asarray(z, dtype=np.uint64).copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(_M1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(_M2)
    z ^= z >> np.uint64(31)
    return z


def keys(seed: int, counters: np.ndarray) -> np.ndarray:
    """64-bit keys for the given counters (uint64 array) of stream ``seed``."""
    c = np.asarray(counters, dtype=np.uint64)
    with np.errstate(over="ignore"):
        state = np.uint64(seed & _MASK64) + (c + np.uint64(1)) * np.uint64(GOLDEN)
        return mix64(state)


def _map_r(k: np.ndarray, scale_exp: int) -> np.ndarray:
    v = (k >> np.uint64(40)).astype(np.int64) - np.int64(1 << 23)
    return np.ldexp(v.astype(np.float32), -23 + scale_exp).astype(np.float32)


def _map_l(k: np.ndarray, scale_exp: int) -> np.ndarray:
    v = (k >> np.uint64(60)).astype(np.int64) - np.int64(8)
    return np.ldexp(v.astype(np.float32), -3 + scale_exp).astype(np.float32)


def _zipf_ranks(k: np.ndarray) -> np.ndarray:
    u = (k >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    e = 1.0 - ZIPF_S
    r = np.floor((1.0 - u * (1.0 - ZIPF_DOMAIN ** e)) ** (1.0 / e))
    r = np.clip(r, 1.0, ZIPF_DOMAIN)
    return r.astype(np.uint64)


def values(seed: int, counters: np.ndarray, mode: str, scale_exp: int = 0) -> np.ndarray:
    """FP32 values for the given counters of stream ``seed`` (host)."""
    k = keys(seed, counters)
    if mode == "R":
        return _map_r(k, scale_exp)
    if mode == "L":
        return _map_l(k, scale_exp)
    if mode == "Z":
        rho = _zipf_ranks(k)
        return _map_r(mix64(rho ^ np.uint64(seed & _MASK64)), scale_exp)
    raise ValueError(f"unknown mode {mode!r}")


def matrix(seed: int, rows: int, cols: int, mode: str, scale_exp: int = 0,
           row_begin: int = 0, row_end: int | None = None,
           chunk_rows: int | None = None) -> np.ndarray:
    """Rows [row_begin, row_end) of the ``rows x cols`` matrix of stream ``seed``."""
    row_end = rows if row_end is None else row_end
    n = row_end - row_begin
    out = np.empty((n, cols), dtype=np.float32)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 22) // max(cols, 1))
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        c = np.arange((row_begin + r0) * cols, (row_begin + r1) * cols, dtype=np.uint64)
        out[r0:r1] = values(seed, c, mode, scale_exp).reshape(r1 - r0, cols)
    return out


def matrix_rows(seed: int, cols: int, row_ids, mode: str, scale_exp: int = 0) -> np.ndarray:
    """The listed rows (any order, repeats allowed) of a ``? x cols`` matrix."""
    row_ids = np.asarray(row_ids, dtype=np.uint64).reshape(-1, 1)
    c = row_ids * np.uint64(cols) + np.arange(cols, dtype=np.uint64).reshape(1, -1)
    return values(seed, c.reshape(-1), mode, scale_exp).reshape(len(row_ids), cols)


def layer_inputs(seed: int, M: int, K: int, N: int, mode: str = "R", bias: bool = False,
                 x_mode: str | None = None):
    """(X[M,K], W[N,K], b[N] or None) for one linear layer, on the host."""
    X = matrix(seed, M, K, x_mode or mode)
    wm = "L" if mode == "L" else "R"
    W = matrix(seed + W_STREAM, N, K, wm, W_SCALE_EXP)
    b = matrix(seed + B_STREAM, 1, N, wm)[0] if bias else None
    return X, W, b


# ----------------------------------------------------------------------------
# device (torch integer ops; bit-identical to the host maps for modes R and L)
# ----------------------------------------------------------------------------
def _s64(c: int) -> int:
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(z, s: int):
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64_torch(z):
    z = z ^ _lsr(z, 30)
    z = z * _s64(_M1)
    z = z ^ _lsr(z, 27)
    z = z * _s64(_M2)
    z = z ^ _lsr(z, 31)
    return z


def matrix_torch(seed: int, rows: int, cols: int, mode: str, scale_exp: int = 0,
                 device="cpu", out=None, chunk_elems: int = 1 << 26):
    """Same matrix as :func:`matrix`, generated with torch ops on ``device``."""
    import torch

    if mode not in ("R", "L"):
        raise ValueError("device generation supports modes R and L only")
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=device)
    flat = out.view(-1)
    total = rows * cols
    for e0 in range(0, total, chunk_elems):
        e1 = min(total, e0 + chunk_elems)
        c = torch.arange(e0 + 1, e1 + 1, dtype=torch.int64, device=device)
        k = _mix64_torch(c * _s64(GOLDEN) + _s64(seed))
        if mode == "R":
            v = _lsr(k, 40) - (1 << 23)
            f = v.to(torch.float32) * float(2.0 ** (-23 + scale_exp))
        else:
            v = _lsr(k, 60) - 8
            f = v.to(torch.float32) * float(2.0 ** (-3 + scale_exp))
        flat[e0:e1] = f
    return out


# ----------------------------------------------------------------------------
# the five benchmark configurations: (M, K, N, seed, x_mode)
# ----------------------------------------------------------------------------
CONFIGS = {
    1: dict(M=100, K=100, N=100, seed=1, x_mode="R"),
    2: dict(M=1000, K=1000, N=1000, seed=2, x_mode="R"),
    3: dict(M=25000, K=4000, N=4000, seed=3, x_mode="R"),
    4: dict(M=25000, K=4000, N=4000, seed=4, x_mode="Z"),
    5: dict(M=200000, K=10000, N=10000, seed=5, x_mode="R"),
}

# Workloads of the transposed layer Y = X^T W (X is [tokens, channels] = K x M, W is K x N).
# "token_mixing_1b": first token-mixing linear of the paper's 1-billion-parameter model
# (Sec. 6.2.1: embedding dimension 4320, token-mixing hidden dimension 8640); 16200 tokens are the
# 721 x 1440 grid of Sec. 3 in 8 x 8 patches.
XTW_CONFIGS = {
    "small": dict(K=200, M=264, N=136, seed=21),
    "token_mixing_1b": dict(K=16200, M=4320, N=8640, seed=22),
}

# Workloads of the mixing MLP (X and Y are [tokens, channels] = M x C, W1 is Hd x C, W2 is C x Hd).
# "channel_mixing_1b": the channel-mixing MLP of the paper's 1-billion-parameter model (Sec. 6.2.1:
# embedding dimension 4320, channel-mixing hidden dimension 4320) over the 16200 tokens of one sample.
# Streams: X seed, W1 seed + 1, b1 seed + 2, W2 seed + 3, b2 seed + 4.
MLP_CONFIGS = {
    "small": dict(M=258, C=264, Hd=136, seed=23),
    "channel_mixing_1b": dict(M=16200, C=4320, Hd=4320, seed=24),
}

# Workload of the patch encoder (a [C, H, W] field -> patches -> linear).  "encoder_1b": the variables
# of Sec. 6 (4 surface + 5 x 13 pressure-level + 3 constant fields = 72) on the 0.25 degree grid cropped
# to 720 x 1440, 8 x 8 patches (16200 tokens of 4608 features) into the 1B model's embedding of 4320.
# The field's element (c, y, x) is element (c * H + y, x) of a (C H) x W matrix of stream `seed`.
ENCODER_CONFIGS = {
    "encoder_1b": dict(C=72, H=720, W=1440, p=8, N=4320, seed=25),
}
