"""Pins for the patch rearrangement of the encoder / decoder (no GPU).

The encoder is a convolution whose kernel equals its stride (Sec. 5 "Encoding and decoding layers");
rearranging the field into non-overlapping patches turns it into the linear layer the rest of the
method works on.  Pinned: the strided convolution written out as six nested loops equals the pinned
forward oracle on the patch matrix; the rearrangement equals the library reshape / transpose that
expresses it; every element appears exactly once; the inverse undoes it; hand-written tiny cases.
"""
import numpy as np
import pytest

import oracle
from paper_2507_05753_amd import inputs


def field_of(seed, C, H, W, mode="L"):
    return inputs.matrix(seed, C * H, W, mode).reshape(C, H, W)


def test_hand_written_case():
    # one channel, 2 x 4 field, 2 x 2 patches: two tokens, rows of the patch matrix read off by eye
    f = np.array([[[0, 1, 2, 3],
                   [4, 5, 6, 7]]], dtype=np.float32)
    assert np.array_equal(oracle.patchify(f, 2), np.array([[0, 1, 4, 5], [2, 3, 6, 7]], dtype=np.float32))
    # two channels: channel-major inside a token
    f2 = np.stack([f[0], f[0] + 10])
    assert np.array_equal(oracle.patchify(f2, 2), np.array([[0, 1, 4, 5, 10, 11, 14, 15],
                                                           [2, 3, 6, 7, 12, 13, 16, 17]], dtype=np.float32))
    # patch size 1: tokens are pixels, features are channels
    assert np.array_equal(oracle.patchify(f2, 1), f2.reshape(2, 8).T)


@pytest.mark.parametrize("C,H,W,p", [(1, 4, 4, 2), (3, 6, 9, 3), (2, 8, 16, 8), (5, 12, 8, 4), (4, 6, 10, 1)])
def test_equals_the_library_reshape_and_is_a_permutation(C, H, W, p):
    f = np.arange(C * H * W, dtype=np.float32).reshape(C, H, W)       # every element distinct
    P = oracle.patchify(f, p)
    want = f.reshape(C, H // p, p, W // p, p).transpose(1, 3, 0, 2, 4).reshape((H // p) * (W // p), C * p * p)
    assert np.array_equal(P, want)
    assert np.array_equal(np.sort(P.reshape(-1)), f.reshape(-1))      # each element exactly once
    assert np.array_equal(oracle.unpatchify(P, C, H, W, p), f)
    # element by element against the index formula
    wp = W // p
    for t in (0, P.shape[0] // 2, P.shape[0] - 1):
        for col in (0, P.shape[1] // 3, P.shape[1] - 1):
            c, rem = divmod(col, p * p)
            dy, dx = divmod(rem, p)
            py, px = divmod(t, wp)
            assert P[t, col] == f[c, py * p + dy, px * p + dx]


@pytest.mark.parametrize("C,H,W,p,N", [(1, 2, 2, 2, 1), (2, 4, 6, 2, 3), (3, 3, 6, 3, 2), (2, 8, 8, 4, 5)])
def test_strided_convolution_is_the_linear_layer_on_patches(C, H, W, p, N):
    f = field_of(41, C, H, W)
    kern = inputs.matrix(42, N * C * p, p, "L").reshape(N, C, p, p)
    b = inputs.matrix(43, 1, N, "L")[0]
    conv = oracle.patch_conv(f, kern, b)                              # six nested loops, lattice values: exact
    lin = oracle.linear(oracle.patchify(f, p), kern.reshape(N, C * p * p), b)
    assert np.array_equal(conv, lin)
    for ways in (2, 4):
        if (C * p * p) % 2 == 0 and N % 2 == 0 and (ways == 2 or ((H // p) * (W // p)) % 2 == 0):
            assert np.array_equal(oracle.jigsaw(ways, oracle.patchify(f, p), kern.reshape(N, C * p * p), b), conv)


def test_argument_checks():
    with pytest.raises(ValueError):
        oracle.patchify(np.zeros((1, 5, 4), np.float32), 2)
    with pytest.raises(ValueError):
        oracle.patchify(np.zeros((1, 4, 6), np.float32), 4)
