"""Pins for the direct-convolution checker (CPU only).

The paper prints no numeric convolution result, so the checker is pinned to what
the definition and the mathematics fix: brute-force dot products, a delta kernel
that must reproduce the zero-padded input, linearity, closed forms, reductions to
a plain matrix product / subsampling / explicit padding, and permutation invariants.
"""
import itertools

import numpy as np
import pytest

from oracle import direct
from paper_2104_04731_amd.inputs import uniform_int8, normal_int8, splitmix64, CONFIGS


def brute(x, w, stride, pad):
    """Independent evaluator: per output, list the in-bounds (input, weight) pairs, sum products."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xl, wl = x.tolist(), w.tolist()
    out = np.zeros((N, K, P, Q), dtype=np.int64)
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        pairs = []
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            h, ww = p * stride + r - pad, q * stride + s - pad
            if 0 <= h < H and 0 <= ww < W:
                pairs.append((xl[n][c][h][ww], wl[k][c][r][s]))
        out[n, k, p, q] = sum(a * b for a, b in pairs)
    return out


TINY = []
_rng = np.random.RandomState(7)
for _ in range(60):
    N = int(_rng.choice([1, 2])); C = int(_rng.choice([1, 3, 5])); K = int(_rng.choice([1, 2, 4]))
    H = int(_rng.randint(1, 10)); W = int(_rng.randint(1, 10))
    pad = int(_rng.randint(0, 4)); stride = int(_rng.randint(1, 4))
    R = int(_rng.randint(1, min(5, H + 2 * pad) + 1)); S = int(_rng.randint(1, min(5, W + 2 * pad) + 1))
    TINY.append((N, C, H, W, K, R, S, stride, pad))
# kernel as large as the padded input (P = Q = 1) and non-dividing strides
TINY += [(1, 2, 3, 4, 2, 5, 6, 1, 1), (2, 1, 7, 5, 1, 3, 2, 3, 0), (1, 3, 1, 1, 2, 1, 1, 2, 0),
         (1, 1, 6, 6, 1, 3, 3, 2, 0), (1, 1, 5, 9, 3, 2, 4, 3, 2)]


@pytest.mark.parametrize("dims", TINY)
def test_brute_force_tiny(dims):
    N, C, H, W, K, R, S, stride, pad = dims
    x = uniform_int8(hash(dims) & 0xFFFF, (N, C, H, W))
    w = uniform_int8((hash(dims) >> 16) & 0xFFFF, (K, C, R, S))
    got = direct.conv2d_int8(x, w, stride, pad)
    assert got.dtype == np.int32
    np.testing.assert_array_equal(got.astype(np.int64), brute(x, w, stride, pad))


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (1, 2), (2, 1), (3, 2)])
def test_delta_kernel_reproduces_padded_input(stride, pad):
    C, H, W, R, S = 3, 7, 9, 3, 4
    x = uniform_int8(11, (2, C, H, W))
    x0 = np.zeros((2, C, H + 2 * pad, W + 2 * pad), np.int32)
    x0[:, :, pad:pad + H, pad:pad + W] = x
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    for r0 in range(R):
        for s0 in range(S):
            w = np.zeros((C, C, R, S), np.int8)
            for k in range(C):
                w[k, k, r0, s0] = 1
            got = direct.conv2d_int8(x, w, stride, pad)
            want = x0[:, :, r0:r0 + stride * (P - 1) + 1:stride, s0:s0 + stride * (Q - 1) + 1:stride]
            np.testing.assert_array_equal(got, want)


def test_delta_centre_is_identity():
    x = uniform_int8(12, (1, 4, 6, 5))
    w = np.zeros((4, 4, 3, 3), np.int8)
    for k in range(4):
        w[k, k, 1, 1] = 1
    np.testing.assert_array_equal(direct.conv2d_int8(x, w, 1, 1), x.astype(np.int32))


def test_linearity():
    sh_x, sh_w = (2, 3, 8, 7), (4, 3, 3, 2)
    a = (uniform_int8(21, sh_x) >> 1); b = (uniform_int8(22, sh_x) >> 1)
    u = (uniform_int8(23, sh_w) >> 1); v = (uniform_int8(24, sh_w) >> 1)
    f = lambda x, w: direct.conv2d_int8(x, w, 2, 1)
    np.testing.assert_array_equal(f((a + b).astype(np.int8), u), f(a, u) + f(b, u))
    np.testing.assert_array_equal(f(a, (u + v).astype(np.int8)), f(a, u) + f(a, v))
    np.testing.assert_array_equal(f((-a).astype(np.int8), u), -f(a, u))


@pytest.mark.parametrize("xv,wv", [(1, 1), (-128, -128), (-128, 127), (127, 127)])
def test_closed_form_constant_tensors(xv, wv):
    N, C, H, W, K, R, S, stride, pad = 1, 5, 9, 8, 2, 3, 4, 1, 2
    x = np.full((N, C, H, W), xv, np.int8); w = np.full((K, C, R, S), wv, np.int8)
    got = direct.conv2d_int8(x, w, stride, pad)
    P, Q = got.shape[2:]
    rows = np.array([sum(0 <= p * stride + r - pad < H for r in range(R)) for p in range(P)])
    cols = np.array([sum(0 <= q * stride + s - pad < W for s in range(S)) for q in range(Q)])
    want = C * xv * wv * rows[:, None] * cols[None, :]
    np.testing.assert_array_equal(got[0, 0], want)
    np.testing.assert_array_equal(got[0, 1], want)
    assert got[0, 0, P // 2, Q // 2] == C * R * S * xv * wv  # interior


def test_pointwise_is_matrix_product():
    x = uniform_int8(31, (2, 24, 5, 6)); w = uniform_int8(32, (7, 24, 1, 1))
    got = direct.conv2d_int8(x, w, 1, 0)
    for n in range(2):
        want = w.reshape(7, 24).astype(np.int64) @ x[n].reshape(24, 30).astype(np.int64)
        np.testing.assert_array_equal(got[n].reshape(7, 30), want)


def test_stride_is_subsampling_and_pad_is_explicit_zero_border():
    x = uniform_int8(41, (1, 3, 11, 13)); w = uniform_int8(42, (2, 3, 3, 5))
    full = direct.conv2d_int8(x, w, 1, 2)
    for st in (2, 3):
        np.testing.assert_array_equal(direct.conv2d_int8(x, w, st, 2), full[:, :, ::st, ::st])
    xz = np.zeros((1, 3, 15, 17), np.int8); xz[:, :, 2:13, 2:15] = x
    np.testing.assert_array_equal(direct.conv2d_int8(xz, w, 1, 0), full)


def test_permutation_invariants():
    x = uniform_int8(51, (2, 6, 7, 7)); w = uniform_int8(52, (5, 6, 3, 3))
    base = direct.conv2d_int8(x, w, 1, 1)
    pc = np.array([3, 0, 5, 1, 4, 2]); pk = np.array([4, 2, 0, 3, 1])
    np.testing.assert_array_equal(
        direct.conv2d_int8(np.ascontiguousarray(x[:, pc]), np.ascontiguousarray(w[:, pc]), 1, 1), base)
    np.testing.assert_array_equal(direct.conv2d_int8(x, np.ascontiguousarray(w[pk]), 1, 1), base[:, pk])


def test_no_flip_and_axis_roles():
    """A kernel that is not symmetric in (r,s): catches a flipped or transposed stencil."""
    x = np.zeros((1, 1, 4, 5), np.int8); x[0, 0, 1, 2] = 1
    w = np.arange(1, 7, dtype=np.int8).reshape(1, 1, 2, 3)
    got = direct.conv2d_int8(x, w, 1, 0)  # P=3, Q=3
    want = np.zeros((3, 3), np.int32)
    for r in range(2):
        for s in range(3):
            p, q = 1 - r, 2 - s
            if 0 <= p < 3 and 0 <= q < 3:
                want[p, q] = w[0, 0, r, s]
    np.testing.assert_array_equal(got[0, 0], want)


def test_rejects_bad_arguments():
    x = np.zeros((1, 1, 2, 2), np.int8); w = np.zeros((1, 1, 3, 3), np.int8)
    with pytest.raises(ValueError):
        direct.conv2d_int8(x, w, 1, 0)


def test_accumulator_headroom_of_all_configs():
    for cfg in CONFIGS.values():
        assert cfg.Kg * 128 * 128 < 2 ** 31


def test_generator_reference_values():
    # SplitMix64 with seed 0: first outputs as published with the algorithm's definition.
    z = splitmix64(0, 3)
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    u = uniform_int8(5, (4096,))
    assert u.min() == -128 and u.max() == 127 and abs(float(u.mean())) < 6
    g = normal_int8(6, (20000,))
    assert 30 < float(g.std()) < 34 and g.min() >= -128 and g.max() <= 127


def test_config_table_matches_definition():
    want = {"C1": (14, 14, 903168), "C2": (56, 56, 231211008), "C3": (112, 112, 944111616),
            "C4a": (14, 14, 3699376128), "C4b": (14, 14, 205520896), "C5": (71, 248, 450764800)}
    for k, (P, Q, ops) in want.items():
        c = CONFIGS[k]
        assert (c.P, c.Q, c.ops) == (P, Q, ops)


# ---- dilated convolution (Sec. 6.1) ---------------------------------------------------------

def brute_dilated(x, w, stride, pad, d):
    """Independent evaluator: per output, list the in-bounds (input, weight) pairs, sum products."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - d * (R - 1) - 1) // stride + 1
    Q = (W + 2 * pad - d * (S - 1) - 1) // stride + 1
    xl, wl = x.tolist(), w.tolist()
    out = np.zeros((N, K, P, Q), dtype=np.int64)
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            h, ww = p * stride + r * d - pad, q * stride + s * d - pad
            if 0 <= h < H and 0 <= ww < W:
                out[n, k, p, q] += xl[n][c][h][ww] * wl[k][c][r][s]
    return out


def spread_kernel(w, d):
    """The stencil blown up with zeros to the dilated access pattern (the paper's own reference
    implementation of a dilated convolution, Sec. 6.1)."""
    K, C, R, S = w.shape
    ws = np.zeros((K, C, d * (R - 1) + 1, d * (S - 1) + 1), dtype=w.dtype)
    ws[:, :, ::d, ::d] = w
    return ws


DILATED_TINY = []
_rng = np.random.RandomState(11)
while len(DILATED_TINY) < 40:
    N = int(_rng.choice([1, 2])); C = int(_rng.choice([1, 2, 3])); K = int(_rng.choice([1, 2, 3]))
    H = int(_rng.randint(3, 12)); W = int(_rng.randint(3, 12))
    R = int(_rng.randint(1, 4)); S = int(_rng.randint(1, 4))
    d = int(_rng.randint(1, 4)); pad = int(_rng.randint(0, 4)); stride = int(_rng.randint(1, 3))
    if d * (R - 1) + 1 <= H + 2 * pad and d * (S - 1) + 1 <= W + 2 * pad:
        DILATED_TINY.append((N, C, H, W, K, R, S, stride, pad, d))


@pytest.mark.parametrize("shape", DILATED_TINY)
def test_dilated_matches_brute_force(shape):
    N, C, H, W, K, R, S, stride, pad, d = shape
    x = uniform_int8(31 + H, (N, C, H, W))
    w = uniform_int8(47 + W, (K, C, R, S))
    np.testing.assert_array_equal(direct.conv2d_int8_dilated(x, w, stride, pad, d), brute_dilated(x, w, stride, pad, d))


@pytest.mark.parametrize("shape", DILATED_TINY[:20] + [(2, 5, 23, 31, 7, 3, 3, 1, 2, 2), (1, 4, 40, 37, 6, 3, 2, 1, 4, 4),
                                                       (1, 3, 30, 30, 4, 5, 5, 2, 6, 3)])
def test_dilated_equals_dense_with_spread_kernel(shape):
    """Pins the dilated loop nest to the (independently pinned) dense one."""
    N, C, H, W, K, R, S, stride, pad, d = shape
    x = uniform_int8(5, (N, C, H, W))
    w = uniform_int8(6, (K, C, R, S))
    np.testing.assert_array_equal(direct.conv2d_int8_dilated(x, w, stride, pad, d),
                                  direct.conv2d_int8(x, spread_kernel(w, d), stride, pad))


def test_dilation_one_is_the_dense_convolution():
    x = uniform_int8(1, (2, 3, 9, 11))
    w = uniform_int8(2, (4, 3, 3, 2))
    for stride, pad in ((1, 0), (2, 1), (1, 2)):
        np.testing.assert_array_equal(direct.conv2d_int8_dilated(x, w, stride, pad, 1), direct.conv2d_int8(x, w, stride, pad))


def test_dilated_delta_kernel_shifts_by_dilation():
    """A kernel that is 1 at tap (r, s) and 0 elsewhere reads the padded input at offset (d*r, d*s)."""
    x = uniform_int8(3, (1, 1, 8, 9))
    d, pad, R, S = 3, 2, 3, 2
    x0 = np.zeros((8 + 2 * pad, 9 + 2 * pad), dtype=np.int32)
    x0[pad:pad + 8, pad:pad + 9] = x[0, 0]
    P, Q = direct.out_hw_dilated(8, 9, R, S, 1, pad, d)
    for r in range(R):
        for s in range(S):
            w = np.zeros((1, 1, R, S), dtype=np.int8)
            w[0, 0, r, s] = 1
            out = direct.conv2d_int8_dilated(x, w, 1, pad, d)
            np.testing.assert_array_equal(out[0, 0], x0[d * r:d * r + P, d * s:d * s + Q])


def test_dilated_rejects_spread_kernel_larger_than_image():
    x = uniform_int8(1, (1, 1, 4, 4))
    w = uniform_int8(2, (1, 1, 3, 3))
    with pytest.raises(ValueError):
        direct.conv2d_int8_dilated(x, w, 1, 0, 2)   # spread extent 5 > 4
