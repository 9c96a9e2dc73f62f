"""TEST INFRASTRUCTURE ONLY: candidate-selection overheads of Sec. 4.4, by definition.

    O_MAC  = MAC_total  - MAC_min
    O_Data = move_total - move_min          (counted in tensor elements, as the paper does)
    score  = w_mac * O_MAC + w_data * O_Data,   minimised over the candidates

Reading of the terms (the paper gives only their names):
  MAC_min    = M*K*C*R*S, the MACs of the definition (M = N*P*Q output pixels).
  MAC_total  = MACs the matrix unit issues once every mapped dimension is padded to
               the unit's extent (Sec. 4.2.4 rule b): ceil(M,x) * ceil(K,y) * depth,
               depth = fused reduction length of the candidate, padded to z.
  move_min   = |in| + |wt| + |out|.
  move_total = every element a layout rewrite reads or writes plus every element the
               GEMM stage reads or writes:
               (|in| + |X'|) + (|wt| + |W'|) + (|X'| + |W'| + |out|)
               with X' the rewritten input and W' the rewritten weights.
Candidates: channel blocks cb in {16,32,64} (pad + split + reorder), a single padded
block cb = ceil(C,16) (pad only), stencil unroll (im2col), and stencil unroll done inside
the GEMM stage (implicit): nothing is rewritten, so X' = in and W' = wt are read once and
O_Data = 0; the unit's pixel extent is filled from one output row at a time and every
kernel row is padded to whole dwords, S4 = ceil(S,4):
               MAC_total = N*P*ceil(Q,x) * ceil(K,y) * ceil(C*R*S4, z).
It is a candidate only inside the domain the interface states for it: padded depth at
most 256, W >= 4, and the input window of one tile -- C*((PT-1)*stride + R) rows of
ceil((QT-1)*stride + S4 + 3, 4) bytes, PT x QT = 1x128 if Q > 64, 2x64 if Q > 32, else
4x32 -- within 40 KB.  A 1x1 kernel over C % 64 == 0 channels takes the layout's second
form (pixels of an image turned into depth-contiguous rows on the fly, weights as they
are): stride 1, no padding, C <= 512, H*W a multiple of 4;
               MAC_total = N*ceil(P*Q,x) * ceil(K,y) * C.
For strides above one, Image Pack (Table 2: the stride phases become channels) followed by
one of the stride-1 layouts on the packed problem is a candidate too.
"""
from __future__ import annotations

PACKED, IM2COL, PAD_ONLY, IMPLICIT, IMAGE_PACK = 1, 2, 3, 4, 5
UNIT_X, UNIT_Y, UNIT_Z = 32, 32, 64  # pixels, output channels, depth


def _ceil(x, m):
    return -(-x // m) * m


def implicit_pointwise(C, R, S):
    """1x1 kernels over whole 64-channel multiples take the second form of the layout."""
    return R == 1 and S == 1 and C % 64 == 0


def implicit_applies(N, C, H, W, K, R, S, stride, pad):
    if implicit_pointwise(C, R, S):
        return stride == 1 and pad == 0 and C <= 512 and (H * W) % 4 == 0
    Q = (W + 2 * pad - S) // stride + 1
    S4 = _ceil(S, 4)
    if _ceil(C * R * S4, UNIT_Z) > 256 or W < 4:
        return False
    PT, QT = (1, 128) if Q > 64 else (2, 64) if Q > 32 else (4, 32)
    rows = (PT - 1) * stride + R
    row_bytes = _ceil((QT - 1) * stride + S4 + 3, 4)
    return max(rows, row_bytes, C * rows * row_bytes) <= 40 * 1024


def candidates(C, dims=None):
    out = [(PACKED, cb) for cb in (64, 32, 16)]
    out.append((IM2COL, 0))
    out.append((PAD_ONLY, _ceil(C, 16)))
    if dims is not None and implicit_applies(*dims):
        out.append((IMPLICIT, 0))
    if dims is not None and dims[7] > 1:                     # Image Pack exists for strides above one
        d2 = image_pack_dims(*dims)
        if d2[1] * d2[5] * d2[6] <= 131072:
            if implicit_applies(*d2):
                out.append((IMAGE_PACK, 0))                  # inner layout: unrolled inside the GEMM stage
            out += [(IMAGE_PACK, cb) for cb in (64, 32, 16)]  # inner layout: channel blocks
    return out


def image_pack_dims(N, C, H, W, K, R, S, stride, pad):
    """The stride-1, pad-0 problem whose channels are the stride phases (Table 2, Image Pack)."""
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    R2, S2 = -(-R // stride), -(-S // stride)
    return (N, C * stride * stride, P + R2 - 1, Q + S2 - 1, K, R2, S2, 1, 0)


def overheads(N, C, H, W, K, R, S, stride, pad, layout, cb):
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    M = N * P * Q
    mac_min = M * K * C * R * S
    if layout == IMAGE_PACK:
        # the packed problem in its inner layout (cb = 0: IMPLICIT, else PACKED with that block); its
        # zero kernel taps count as overhead against the original definition; the pack itself writes
        # X2 and W2, which the inner stage reads again
        d2 = image_pack_dims(N, C, H, W, K, R, S, stride, pad)
        o_mac, o_data, rewritten = overheads(*d2, IMPLICIT if cb == 0 else PACKED, cb)
        x2 = d2[0] * d2[1] * d2[2] * d2[3]
        w2 = K * d2[1] * d2[5] * d2[6]
        return o_mac + M * K * d2[1] * d2[5] * d2[6] - mac_min, o_data + 2 * (x2 + w2), rewritten + x2 + w2
    if layout == IMPLICIT:
        if implicit_pointwise(C, R, S):
            return N * _ceil(P * Q, UNIT_X) * _ceil(K, UNIT_Y) * C - mac_min, 0, 0
        depth = _ceil(C * R * _ceil(S, 4), UNIT_Z)
        return N * P * _ceil(Q, UNIT_X) * _ceil(K, UNIT_Y) * depth - mac_min, 0, 0
    if layout == IM2COL:
        depth = _ceil(C * R * S, UNIT_Z)
        x_elems = M * depth
    else:
        cpad = _ceil(C, cb)
        depth = _ceil(cpad * R * S, UNIT_Z)
        x_elems = N * cpad * (H + 2 * pad) * (W + 2 * pad)
    w_elems = K * depth
    mac_total = _ceil(M, UNIT_X) * _ceil(K, UNIT_Y) * depth
    o_mac = mac_total - mac_min
    o_data = 2 * x_elems + 2 * w_elems
    return o_mac, o_data, x_elems + w_elems


def select(N, C, H, W, K, R, S, stride, pad, w_mac, w_data):
    """Return (layout, cb, score) of the cheapest candidate.

    Ties: fewer rewritten elements, then lower layout code, then larger block."""
    best = None
    for layout, cb in candidates(C, (N, C, H, W, K, R, S, stride, pad)):
        o_mac, o_data, ws = overheads(N, C, H, W, K, R, S, stride, pad, layout, cb)
        score = w_mac * o_mac + w_data * o_data
        key = (score, ws, layout, -cb)
        if best is None or key < best[0]:
            best = (key, layout, cb, score)
    return best[1], best[2], best[3]
