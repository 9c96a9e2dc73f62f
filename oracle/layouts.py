"""TEST INFRASTRUCTURE ONLY: the layout rewrites and the GEMM unit, by definition.

Each function is the index map of the corresponding rewrite written out with
numpy slicing; no blocking or fusion beyond what the map itself states.

  pack_layout   Table 2 rows Pad, Split, Reorder applied to the input (the
                reference mapping of Sec. 5.1: the channel dimension is padded to
                a multiple of the block, split, and the block moved innermost);
                the spatial zero border of the convolution is materialised too.
  pack_weights  the same rewrites on the weights, then Fuse (Table 2 row 5) of the
                reduction dimensions into one GEMM depth, zero-padded to `kalign`
                (for the stencil unroll done inside the GEMM stage: every kernel row
                first padded to a multiple of four taps).
  im2col        Stencil Unroll + Fuse (Table 2 rows 1 and 5; "im2col" in Sec. 6.2).
  gemm_nt       the matrix unit of Sec. 5.1: C[x][y] += sum_z A[x][z] * B[y][z].
  image_pack    Image Pack of Table 2 (row 1, the alternative to Stencil Unroll for strides
                above one: [N, I] => [N*s, I/s] with the access function unchanged): the s*s
                stride phases of the padded image become channels, and a stride-s convolution
                becomes a stride-1 convolution with the kernel phase-split the same way.
"""
from __future__ import annotations

import numpy as np


def ceil_to(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def pack_layout(x: np.ndarray, cb: int, pad: int) -> np.ndarray:
    """[N,C,H,W] -> [N, ceil(C/cb), H+2pad, W+2pad, cb]; zeros for c >= C and the border."""
    N, C, H, W = x.shape
    Cb = (C + cb - 1) // cb
    y = np.zeros((N, Cb, H + 2 * pad, W + 2 * pad, cb), dtype=x.dtype)
    for c in range(C):
        y[:, c // cb, pad:pad + H, pad:pad + W, c % cb] = x[:, c]
    return y


def pack_layout_nhwc(x: np.ndarray, cb: int, pad: int) -> np.ndarray:
    """The same rewrite from an NHWC source (Sec. 5.2: the free dimensions of the source may be in any
    order): [N,H,W,C] -> [N, ceil(C/cb), H+2pad, W+2pad, cb]; y[n][c//cb][h+pad][w+pad][c%cb] = x[n][h][w][c]."""
    N, H, W, C = x.shape
    Cb = (C + cb - 1) // cb
    y = np.zeros((N, Cb, H + 2 * pad, W + 2 * pad, cb), dtype=x.dtype)
    for c in range(C):
        y[:, c // cb, pad:pad + H, pad:pad + W, c % cb] = x[:, :, :, c]
    return y


def packed_depth(C: int, R: int, S: int, cb: int, kalign: int = 64) -> int:
    return ceil_to(((C + cb - 1) // cb) * R * S * cb, kalign)


def pack_weights_blocked(w: np.ndarray, cb: int, kalign: int = 64) -> np.ndarray:
    """[K,C,R,S] -> [K, depth]; depth index j = ((c//cb * R + r) * S + s) * cb + c%cb."""
    K, C, R, S = w.shape
    y = np.zeros((K, packed_depth(C, R, S, cb, kalign)), dtype=w.dtype)
    for c in range(C):
        for r in range(R):
            for s in range(S):
                j = ((c // cb * R + r) * S + s) * cb + c % cb
                y[:, j] = w[:, c, r, s]
    return y


def pack_weights_im2col(w: np.ndarray, kalign: int = 64) -> np.ndarray:
    """[K,C,R,S] -> [K, depth]; depth index j = (c*R + r)*S + s, zero-padded."""
    K, C, R, S = w.shape
    y = np.zeros((K, ceil_to(C * R * S, kalign)), dtype=w.dtype)
    y[:, :C * R * S] = w.reshape(K, C * R * S)
    return y


def pack_weights_implicit(w: np.ndarray, kalign: int = 64) -> np.ndarray:
    """[K,C,R,S] -> [K, depth]; depth index j = (c*R + r)*S4 + s with S4 = ceil(S,4), zero-padded."""
    K, C, R, S = w.shape
    if R == 1 and S == 1 and C % 64 == 0:   # 1x1 over whole 64-channel multiples: [K][C] as it is
        return w.reshape(K, C).copy()
    S4 = ceil_to(S, 4)
    y = np.zeros((K, C * R, S4), dtype=w.dtype)
    y[:, :, :S] = w.reshape(K, C * R, S)
    out = np.zeros((K, ceil_to(C * R * S4, kalign)), dtype=w.dtype)
    out[:, :C * R * S4] = y.reshape(K, C * R * S4)
    return out


def im2col(x: np.ndarray, R: int, S: int, stride: int, pad: int,
           kalign: int = 64) -> np.ndarray:
    """[N,C,H,W] -> [N*P*Q, depth]; A[(n,p,q)][(c,r,s)] = x0[n][c][p*st+r-pad][q*st+s-pad]."""
    N, C, H, W = x.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    x0 = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=x.dtype)
    x0[:, :, pad:pad + H, pad:pad + W] = x
    A = np.zeros((N, P, Q, ceil_to(C * R * S, kalign)), dtype=x.dtype)
    for c in range(C):
        for r in range(R):
            for s in range(S):
                A[:, :, :, (c * R + r) * S + s] = \
                    x0[:, c, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
    return A.reshape(N * P * Q, -1)


def gemm_nt(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C[x][y] = sum_z A[x][z] * B[y][z], int8 operands, exact, returned as int32."""
    C = A.astype(np.int64) @ B.astype(np.int64).T
    assert np.all(np.abs(C) < 2 ** 31)
    return C.astype(np.int32)


def image_pack_dims(N, C, H, W, K, R, S, stride, pad):
    """The stride-1, pad-0 problem an image-packed convolution turns into."""
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    R2, S2 = -(-R // stride), -(-S // stride)
    return (N, C * stride * stride, P + R2 - 1, Q + S2 - 1, K, R2, S2, 1, 0)


def image_pack(x: np.ndarray, R: int, S: int, stride: int, pad: int) -> np.ndarray:
    """[N,C,H,W] -> [N, C*s*s, H2, W2]; X2[n][(c*s + a)*s + b][i][j] = x0[n][c][s*i + a][s*j + b]
    with x0 the zero-padded image continued by zeros."""
    N, C, H, W = x.shape
    s = stride
    _, C2, H2, W2, _, _, _, _, _ = image_pack_dims(N, C, H, W, 1, R, S, stride, pad)
    x0 = np.zeros((N, C, max(H + 2 * pad, s * H2), max(W + 2 * pad, s * W2)), dtype=x.dtype)
    x0[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, C2, H2, W2), dtype=x.dtype)
    for c in range(C):
        for a in range(s):
            for b in range(s):
                y[:, (c * s + a) * s + b] = x0[:, c, a:a + s * H2:s, b:b + s * W2:s]
    return y


def image_pack_weights(w: np.ndarray, stride: int) -> np.ndarray:
    """[K,C,R,S] -> [K, C*s*s, ceil(R/s), ceil(S/s)]; W2[k][(c*s + a)*s + b][r][t] = w[k][c][s*r + a][s*t + b],
    zero where s*r + a >= R or s*t + b >= S."""
    K, C, R, S = w.shape
    s = stride
    R2, S2 = -(-R // s), -(-S // s)
    w0 = np.zeros((K, C, s * R2, s * S2), dtype=w.dtype)
    w0[:, :, :R, :S] = w
    y = np.zeros((K, C * s * s, R2, S2), dtype=w.dtype)
    for c in range(C):
        for a in range(s):
            for b in range(s):
                y[:, (c * s + a) * s + b] = w0[:, c, a::s, b::s]
    return y


def unpack_nhwc(out: np.ndarray) -> np.ndarray:
    """Tensor unpacking for an NHWC consumer (Sec. 5.1 benchmark step, Sec. 5.2 layout):
    [N,K,P,Q] -> [N,P,Q,K]; y[n][p][q][k] = out[n][k][p][q]."""
    N, K, P, Q = out.shape
    y = np.zeros((N, P, Q, K), dtype=out.dtype)
    for k in range(K):
        y[:, :, :, k] = out[:, k]
    return y


def requant(x: np.ndarray, shift: int, relu: bool) -> np.ndarray:
    """Activation between two int8 layers, as the accelerator's ALU does it (Sec. 5.1: shift, min, max
    on the 32-bit accumulator): rounding right shift (half rounds towards +infinity),
    optional max(., 0), then clipping to int8.  y = clip(relu(floor(x / 2^shift + 1/2)), -128, 127)."""
    assert 0 <= shift <= 31
    v = x.astype(np.int64)
    if shift > 0:
        v = (v + (1 << (shift - 1))) >> shift     # arithmetic shift = floor division by 2^shift
    if relu:
        v = np.maximum(v, 0)
    return np.clip(v, -128, 127).astype(np.int8)


def dilation_dims(N, C, H, W, K, R, S, pad, dilation):
    """The dense stride-1, pad-0 problem a dilated stride-1 convolution turns into (Sec. 6.1; Table 2
    row 1, Image Pack [N, I] => [N*s, I/s] on both image axes): d*d sub-images per image."""
    d = dilation
    return (N * d * d, C, -(-(H + 2 * pad) // d), -(-(W + 2 * pad) // d), K, R, S, 1, 0)


def dilation_pack(x: np.ndarray, pad: int, dilation: int) -> np.ndarray:
    """[N,C,H,W] -> [N*d*d, C, H2, W2]; X2[(n*d + a)*d + b][c][i][j] = x0[n][c][d*i + a][d*j + b] with x0
    the zero-padded image continued by zeros: sub-image (a, b) holds the pixels whose padded row is a
    and whose padded column is b modulo d, the only ones one output pixel of that phase ever reads."""
    N, C, H, W = x.shape
    d = dilation
    H2, W2 = -(-(H + 2 * pad) // d), -(-(W + 2 * pad) // d)
    x0 = np.zeros((N, C, d * H2, d * W2), dtype=x.dtype)
    x0[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N * d * d, C, H2, W2), dtype=x.dtype)
    for n in range(N):
        for a in range(d):
            for b in range(d):
                y[(n * d + a) * d + b] = x0[n, :, a::d, b::d]
    return y


def dilation_unpack(o2: np.ndarray, dilation: int, P: int, Q: int) -> np.ndarray:
    """Interleaving the sub-images' results back (Sec. 6.1): [N*d*d, K, P2, Q2] -> [N, K, P, Q];
    out[n][k][d*i + a][d*j + b] = O2[(n*d + a)*d + b][k][i][j] for d*i + a < P, d*j + b < Q."""
    d = dilation
    N2, K, P2, Q2 = o2.shape
    N = N2 // (d * d)
    out = np.zeros((N, K, P, Q), dtype=o2.dtype)
    for n in range(N):
        for a in range(d):
            for b in range(d):
                sub = out[n, :, a::d, b::d]
                sub[...] = o2[(n * d + a) * d + b][:, :sub.shape[1], :sub.shape[2]]
    return out


def im2col_nhwc(xh: np.ndarray, R: int, S: int, stride: int, pad: int, kalign: int = 64) -> np.ndarray:
    """Stencil Unroll + Fuse from an NHWC source (Sec. 5.2: the source layout decides what a rewrite costs):
    [N,H,W,C] -> [N*P*Q, depth]; A[(n,p,q)][(r*S + s)*C + c] = x0[n][p*st+r-pad][q*st+s-pad][c] -- the
    channels of a tap stay contiguous, so every tap is one run of C source bytes."""
    N, H, W, C = xh.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    x0 = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=xh.dtype)
    x0[:, pad:pad + H, pad:pad + W, :] = xh
    A = np.zeros((N, P, Q, ceil_to(C * R * S, kalign)), dtype=xh.dtype)
    for r in range(R):
        for s in range(S):
            A[:, :, :, (r * S + s) * C:(r * S + s + 1) * C] = \
                x0[:, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride, :]
    return A.reshape(N * P * Q, -1)


def pack_weights_rsc(w: np.ndarray, kalign: int = 64) -> np.ndarray:
    """[K,C,R,S] -> [K][depth], depth index (r*S + s)*C + c (the order im2col_nhwc unrolls in), zero-padded."""
    K, C, R, S = w.shape
    y = np.zeros((K, ceil_to(C * R * S, kalign)), dtype=w.dtype)
    for r in range(R):
        for s in range(S):
            y[:, (r * S + s) * C:(r * S + s + 1) * C] = w[:, :, r, s]
    return y
