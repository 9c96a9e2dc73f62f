"""Pins for the layout-rewrite and GEMM-unit definitions (CPU only).

The rewrites are pinned against the independently written direct convolution:
a rewritten operand pair, pushed through the matrix unit's definition, must give the
convolution itself.  Element-wise brute force, round trips and zero counts pin the rest.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import direct, layouts
from paper_2104_04731_amd.inputs import uniform_int8, CONFIGS

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_gemm_unit_hand_example():
    want = np.loadtxt(os.path.join(GOLD, "gemm_unit_1x16x16.txt"), dtype=np.int64).reshape(1, 16)
    A = np.arange(1, 17, dtype=np.int8).reshape(1, 16)
    B = np.array([[y - z for z in range(16)] for y in range(16)], dtype=np.int8)
    np.testing.assert_array_equal(layouts.gemm_nt(A, B), want)
    np.testing.assert_array_equal(want[0], 136 * np.arange(16) - 1360)


def test_gemm_unit_is_b_transposed_and_signed():
    A = np.array([[-128, 127, 3]], np.int8); B = np.array([[-128, -128, 0], [1, 2, 3]], np.int8)
    np.testing.assert_array_equal(layouts.gemm_nt(A, B), [[16384 - 16256, -128 + 254 + 9]])


@pytest.mark.parametrize("cb,pad", [(4, 0), (16, 1), (16, 3), (32, 2), (64, 1)])
def test_pack_layout_elementwise(cb, pad):
    N, C, H, W = 2, 37, 5, 6
    x = uniform_int8(61, (N, C, H, W))
    y = layouts.pack_layout(x, cb, pad)
    Cb = -(-C // cb)
    assert y.shape == (N, Cb, H + 2 * pad, W + 2 * pad, cb)
    yl, xl = y.tolist(), x.tolist()
    for n, b, hp, wp, i in itertools.product(range(N), range(Cb), range(H + 2 * pad), range(W + 2 * pad), range(cb)):
        c, h, w = b * cb + i, hp - pad, wp - pad
        want = xl[n][c][h][w] if (c < C and 0 <= h < H and 0 <= w < W) else 0
        assert yl[n][b][hp][wp][i] == want
    # round trip: un-reorder, un-split, crop
    back = y.transpose(0, 1, 4, 2, 3).reshape(N, Cb * cb, H + 2 * pad, W + 2 * pad)
    np.testing.assert_array_equal(back[:, :C, pad:pad + H, pad:pad + W], x)


@pytest.mark.parametrize("name", ["C1", "C2", "C4b"])
def test_im2col_then_gemm_is_the_convolution(name):
    cfg = CONFIGS[name]; x, w = cfg.make()
    A = layouts.im2col(x, cfg.R, cfg.S, cfg.stride, cfg.pad)
    B = layouts.pack_weights_im2col(w)
    assert A.shape == (cfg.M, -(-cfg.Kg // 64) * 64) and B.shape == (cfg.K, A.shape[1])
    got = layouts.gemm_nt(B, A).reshape(cfg.K, cfg.N, cfg.P, cfg.Q).transpose(1, 0, 2, 3)
    np.testing.assert_array_equal(got, direct.conv2d_int8(x, w, cfg.stride, cfg.pad))


def test_im2col_elementwise_small():
    N, C, H, W, R, S, st, pad = 2, 3, 6, 7, 3, 2, 2, 1
    x = uniform_int8(62, (N, C, H, W)); xl = x.tolist()
    A = layouts.im2col(x, R, S, st, pad)
    P = (H + 2 * pad - R) // st + 1; Q = (W + 2 * pad - S) // st + 1
    assert A.shape == (N * P * Q, 64)
    for n, p, q, c, r, s in itertools.product(range(N), range(P), range(Q), range(C), range(R), range(S)):
        h, w = p * st + r - pad, q * st + s - pad
        want = xl[n][c][h][w] if (0 <= h < H and 0 <= w < W) else 0
        assert A[(n * P + p) * Q + q, (c * R + r) * S + s] == want
    assert not A[:, C * R * S:].any()


@pytest.mark.parametrize("dims,cb", [((2, 5, 6, 7, 3, 3, 2, 1, 1), 16), ((1, 40, 5, 5, 6, 3, 3, 2, 1), 16),
                                     ((1, 40, 5, 5, 6, 3, 3, 1, 2), 32), ((1, 70, 4, 6, 5, 1, 1, 1, 0), 64),
                                     ((1, 3, 9, 9, 4, 7, 7, 2, 3), 16), ((1, 33, 4, 4, 2, 2, 3, 1, 0), 48)])
def test_blocked_operands_give_the_convolution(dims, cb):
    """Implicit GEMM by definition over the packed operands == direct convolution."""
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(63, (N, C, H, W)); w = uniform_int8(64, (K, C, R, S))
    X = layouts.pack_layout(x, cb, pad); Wq = layouts.pack_weights_blocked(w, cb)
    Cb = X.shape[1]
    assert Wq.shape == (K, layouts.packed_depth(C, R, S, cb)) and Wq.shape[1] % 64 == 0
    P = (H + 2 * pad - R) // st + 1; Q = (W + 2 * pad - S) // st + 1
    A = np.zeros((N, P, Q, Wq.shape[1]), np.int8)
    for b, r, s in itertools.product(range(Cb), range(R), range(S)):
        j = ((b * R + r) * S + s) * cb
        A[:, :, :, j:j + cb] = X[:, b, r:r + st * (P - 1) + 1:st, s:s + st * (Q - 1) + 1:st, :]
    got = layouts.gemm_nt(Wq, A.reshape(N * P * Q, -1)).reshape(K, N, P, Q).transpose(1, 0, 2, 3)
    np.testing.assert_array_equal(got, direct.conv2d_int8(x, w, st, pad))
    # everything that is not a true weight is zero
    assert np.count_nonzero(Wq) == np.count_nonzero(w)


def test_weight_pack_im2col_is_row_padded_copy():
    w = uniform_int8(65, (5, 3, 7, 7))
    B = layouts.pack_weights_im2col(w)
    assert B.shape == (5, 192)
    np.testing.assert_array_equal(B[:, :147], w.reshape(5, 147))
    assert not B[:, 147:].any()


@pytest.mark.parametrize("dims", [(2, 3, 9, 9, 4, 7, 7, 2, 3), (1, 1, 23, 12, 3, 20, 5, 2, 0),
                                  (1, 5, 6, 8, 2, 3, 3, 1, 1), (1, 2, 5, 7, 3, 1, 1, 1, 0), (1, 3, 6, 9, 2, 2, 9, 3, 2)])
def test_row_padded_weights_give_the_convolution(dims):
    """Stencil unroll in the depth order (c, r, s') with kernel rows padded to four taps: the GEMM of
    the padded weights with the matching unrolled input (padded taps read whatever lies right of
    the window -- here the next real columns or zero -- and meet zero weights) == direct convolution."""
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(66, (N, C, H, W)); w = uniform_int8(67, (K, C, R, S))
    B = layouts.pack_weights_implicit(w)
    S4 = -(-S // 4) * 4
    assert B.shape == (K, -(-C * R * S4 // 64) * 64)
    P = (H + 2 * pad - R) // st + 1; Q = (W + 2 * pad - S) // st + 1
    x0 = np.zeros((N, C, H + 2 * pad, W + 2 * pad + S4), np.int8)      # room right of the last window
    x0[:, :, pad:pad + H, pad:pad + W] = x
    x0[:, :, :, W + 2 * pad:] = 77                                       # must not matter
    A = np.zeros((N, P, Q, B.shape[1]), np.int8)
    for c, r, s in itertools.product(range(C), range(R), range(S4)):
        A[:, :, :, (c * R + r) * S4 + s] = x0[:, c, r:r + st * (P - 1) + 1:st, s:s + st * (Q - 1) + 1:st]
    got = layouts.gemm_nt(B, A.reshape(N * P * Q, -1)).reshape(K, N, P, Q).transpose(1, 0, 2, 3)
    np.testing.assert_array_equal(got, direct.conv2d_int8(x, w, st, pad))
    # the true weights, each once, in (c, r, s) order; zeros elsewhere
    assert np.count_nonzero(B) == np.count_nonzero(w)
    np.testing.assert_array_equal(B[:, :C * R * S4].reshape(K, C * R, S4)[:, :, :S].reshape(K, C, R, S), w)


def test_pointwise_weights_are_the_weights():
    w = uniform_int8(68, (5, 128, 1, 1))
    np.testing.assert_array_equal(layouts.pack_weights_implicit(w), w.reshape(5, 128))
    assert layouts.pack_weights_implicit(uniform_int8(69, (5, 32, 1, 1))).shape == (5, 128)   # 32 channels: padded taps


@pytest.mark.parametrize("dims", [(2, 3, 9, 9, 4, 7, 7, 2, 3), (1, 1, 23, 12, 3, 20, 5, 2, 0), (1, 2, 10, 11, 3, 3, 3, 3, 1),
                                  (1, 4, 8, 8, 2, 2, 2, 2, 0), (2, 2, 7, 9, 3, 1, 1, 2, 0), (1, 3, 12, 10, 2, 5, 4, 3, 2),
                                  (1, 2, 6, 6, 2, 3, 3, 1, 1), (1, 1, 9, 9, 1, 4, 4, 4, 0)])
def test_image_pack_turns_a_strided_convolution_into_a_dense_one(dims):
    """Image Pack (Table 2): stride phases become channels; the stride-1 convolution of the packed
    image with the phase-split kernel is the strided convolution."""
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(70, (N, C, H, W)); w = uniform_int8(71, (K, C, R, S))
    x2 = layouts.image_pack(x, R, S, st, pad); w2 = layouts.image_pack_weights(w, st)
    d2 = layouts.image_pack_dims(*dims)
    assert x2.shape == d2[:4] and w2.shape == (K, d2[1], d2[5], d2[6]) and d2[7:] == (1, 0)
    np.testing.assert_array_equal(direct.conv2d_int8(x2, w2, 1, 0), direct.conv2d_int8(x, w, st, pad))
    # every weight appears exactly once; the packed image holds every input byte a window can touch
    assert np.count_nonzero(w2) == np.count_nonzero(w)
    assert sorted(np.abs(w2[w2 != 0]).tolist()) == sorted(np.abs(w[w != 0]).tolist())


def test_image_pack_elementwise_small():
    N, C, H, W, R, S, st, pad = 1, 2, 7, 8, 3, 5, 2, 1
    x = (np.arange(N * C * H * W) % 120 + 1).astype(np.int8).reshape(N, C, H, W); xl = x.tolist()
    y = layouts.image_pack(x, R, S, st, pad)
    _, C2, H2, W2 = y.shape
    assert (C2, H2, W2) == (C * 4, 4 + 2 - 1, 3 + 3 - 1)       # P=4, Q=3, R2=2, S2=3
    for c, a, b, i, j in itertools.product(range(C), range(st), range(st), range(H2), range(W2)):
        h, wcol = st * i + a - pad, st * j + b - pad
        want = xl[0][c][h][wcol] if (0 <= h < H and 0 <= wcol < W) else 0
        assert y[0, (c * st + a) * st + b, i, j] == want


def test_pack_layout_from_nhwc_source():
    """Same destination as from NCHW: only the source's dimension order differs; element by element too."""
    N, C, H, W, cb, pad = 2, 37, 4, 5, 16, 1
    x = uniform_int8(72, (N, C, H, W))
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    y = layouts.pack_layout_nhwc(xh, cb, pad)
    np.testing.assert_array_equal(y, layouts.pack_layout(x, cb, pad))
    xl = xh.tolist(); Cb = -(-C // cb)
    for n, b, hp, wp, i in itertools.product(range(N), range(Cb), range(H + 2 * pad), range(W + 2 * pad), range(cb)):
        c, h, w = b * cb + i, hp - pad, wp - pad
        want = xl[n][h][w][c] if (c < C and 0 <= h < H and 0 <= w < W) else 0
        assert y[n][b][hp][wp][i] == want


def test_unpack_nhwc_elementwise():
    o = (np.arange(2 * 5 * 3 * 4, dtype=np.int32) * 7919 - 100000).reshape(2, 5, 3, 4)
    y = layouts.unpack_nhwc(o)
    assert y.shape == (2, 3, 4, 5)
    ol = o.tolist()
    for n, k, p, q in itertools.product(range(2), range(5), range(3), range(4)):
        assert y[n, p, q, k] == ol[n][k][p][q]


def test_requant_against_exact_rational_arithmetic():
    """floor(x / 2^s + 1/2) computed with Python integers and Fractions, every case of sign and tie."""
    from fractions import Fraction
    import math
    xs = [0, 1, -1, 2, -2, 3, -3, 7, 8, -8, 9, 127, 128, 129, -127, -128, -129, 255, 256, -255, -256, 1000, -1000,
          16383, 16384, -16384, 37748736, -37748736, 2 ** 31 - 1, -2 ** 31]
    xs += [v * 8 + d for v in range(-20, 21) for d in (-4, -3, 0, 3, 4, 5)]       # ties at shift 3: d = +-4
    x = np.array(xs, dtype=np.int32)
    for shift in (0, 1, 3, 4, 8, 17, 31):
        for relu in (False, True):
            got = layouts.requant(x, shift, relu).tolist()
            for v, g in zip(xs, got):
                r = math.floor(Fraction(v, 2 ** shift) + Fraction(1, 2))
                if relu:
                    r = max(r, 0)
                assert g == min(max(r, -128), 127), (v, shift, relu)
    # monotone, and the identity on int8 values when nothing is shifted
    ramp = np.arange(-70000, 70000, 7, dtype=np.int32)
    for shift in (0, 5, 9):
        y = layouts.requant(ramp, shift, False).astype(np.int32)
        assert np.all(np.diff(y) >= 0)
    small = np.arange(-128, 128, dtype=np.int32)
    np.testing.assert_array_equal(layouts.requant(small, 0, False), small.astype(np.int8))
    np.testing.assert_array_equal(layouts.requant(small, 0, True), np.maximum(small, 0).astype(np.int8))
    assert layouts.requant(np.array([4, -4, 12, -12], np.int32), 3, False).tolist() == [1, 0, 2, -1]   # ties go up


# ---- dilation as Image Pack into the batch (Sec. 6.1, Table 2 row 1) ---------------------------

DILATION_SHAPES = [
    # N, C, H, W, K, R, S, pad, d
    (1, 1, 7, 7, 1, 3, 3, 0, 2),
    (2, 3, 9, 10, 4, 3, 3, 2, 2),
    (1, 2, 11, 8, 3, 2, 3, 3, 3),
    (1, 4, 13, 17, 2, 3, 3, 4, 4),
    (2, 1, 6, 5, 2, 1, 1, 1, 2),
    (1, 2, 10, 10, 2, 3, 1, 0, 3),
]


@pytest.mark.parametrize("shape", DILATION_SHAPES)
def test_dilation_pack_conv_unpack_is_the_dilated_convolution(shape):
    N, C, H, W, K, R, S, pad, d = shape
    x = uniform_int8(21, (N, C, H, W))
    w = uniform_int8(22, (K, C, R, S))
    want = direct.conv2d_int8_dilated(x, w, 1, pad, d)
    N2, C2, H2, W2, K2, R2, S2, st2, pad2 = layouts.dilation_dims(N, C, H, W, K, R, S, pad, d)
    x2 = layouts.dilation_pack(x, pad, d)
    assert x2.shape == (N2, C2, H2, W2) and (K2, R2, S2, st2, pad2) == (K, R, S, 1, 0)
    o2 = direct.conv2d_int8(x2, w, 1, 0)
    got = layouts.dilation_unpack(o2, d, want.shape[2], want.shape[3])
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("shape", DILATION_SHAPES[:4])
def test_dilation_pack_element_by_element(shape):
    N, C, H, W, K, R, S, pad, d = shape
    x = uniform_int8(23, (N, C, H, W))
    x2 = layouts.dilation_pack(x, pad, d)
    H2, W2 = x2.shape[2], x2.shape[3]
    for n2, c, i, j in itertools.product(range(N * d * d), range(C), range(H2), range(W2)):
        n, a, b = n2 // (d * d), (n2 // d) % d, n2 % d
        h, ww = d * i + a - pad, d * j + b - pad
        want = int(x[n, c, h, ww]) if 0 <= h < H and 0 <= ww < W else 0
        assert int(x2[n2, c, i, j]) == want


def test_dilation_pack_keeps_every_input_element_once():
    x = np.arange(1, 2 * 3 * 5 * 7 + 1, dtype=np.int64).reshape(2, 3, 5, 7)
    x2 = layouts.dilation_pack(x, 1, 3)
    vals = np.sort(x2[x2 != 0])
    np.testing.assert_array_equal(vals, np.arange(1, x.size + 1))


def test_dilation_unpack_element_by_element():
    d, N, K, P, Q = 3, 2, 2, 7, 8
    P2, Q2 = 4, 3   # larger than ceil(P/d), ceil(Q/d) = 3, 3 in one axis: surplus rows are dropped
    o2 = np.arange(N * d * d * K * P2 * Q2, dtype=np.int32).reshape(N * d * d, K, P2, Q2)
    out = layouts.dilation_unpack(o2, d, P, Q)
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        assert out[n, k, p, q] == o2[(n * d + p % d) * d + q % d, k, p // d, q // d]


# ---- stencil unrolling from an NHWC source (Sec. 5.2) --------------------------------------------------------
@pytest.mark.parametrize("dims", [(2, 3, 6, 7, 4, 3, 2, 2, 1), (1, 16, 9, 9, 5, 3, 3, 1, 1), (1, 5, 8, 6, 3, 1, 1, 2, 0),
                                  (2, 20, 5, 11, 7, 5, 3, 1, 2), (1, 64, 7, 7, 8, 3, 3, 1, 1)], ids=str)
def test_im2col_nhwc_then_gemm_is_the_convolution(dims):
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(81, (N, C, H, W)); w = uniform_int8(82, (K, C, R, S))
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    A = layouts.im2col_nhwc(xh, R, S, st, pad)
    B = layouts.pack_weights_rsc(w)
    want = direct.conv2d_int8(x, w, st, pad)
    P, Q = want.shape[2], want.shape[3]
    assert A.shape == (N * P * Q, -(-C * R * S // 64) * 64) and B.shape == (K, A.shape[1])
    got = layouts.gemm_nt(B, A).reshape(K, N, P, Q).transpose(1, 0, 2, 3)
    np.testing.assert_array_equal(got, want)


def test_im2col_nhwc_elementwise_small_and_against_the_nchw_form():
    N, C, H, W, R, S, st, pad = 2, 3, 6, 7, 3, 2, 2, 1
    x = uniform_int8(83, (N, C, H, W)); xl = x.tolist()
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    A = layouts.im2col_nhwc(xh, R, S, st, pad)
    P = (H + 2 * pad - R) // st + 1; Q = (W + 2 * pad - S) // st + 1
    for n, p, q, c, r, s in itertools.product(range(N), range(P), range(Q), range(C), range(R), range(S)):
        h, ww = p * st + r - pad, q * st + s - pad
        want = xl[n][c][h][ww] if (0 <= h < H and 0 <= ww < W) else 0
        assert A[(n * P + p) * Q + q, (r * S + s) * C + c] == want
    assert not A[:, C * R * S:].any()
    # the same matrix as the NCHW form, with its depth columns permuted (c, r, s) -> (r, s, c)
    A0 = layouts.im2col(x, R, S, st, pad)
    perm = [(c * R + r) * S + s for r in range(R) for s in range(S) for c in range(C)]
    np.testing.assert_array_equal(A[:, :C * R * S], A0[:, perm])


def test_pack_weights_rsc_is_a_permutation_of_the_kernel():
    w = np.arange(1, 2 * 3 * 2 * 4 + 1, dtype=np.int64).reshape(2, 3, 2, 4)
    y = layouts.pack_weights_rsc(w)
    assert y.shape == (2, 64) and not y[:, 24:].any()
    for k, c, r, s in itertools.product(range(2), range(3), range(2), range(4)):
        assert y[k, (r * 4 + s) * 3 + c] == w[k, c, r, s]
