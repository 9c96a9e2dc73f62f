"""TEST INFRASTRUCTURE ONLY: candidate selection of Sec. 4.4, by definition.

    O_MAC  = MAC_total  - MAC_min
    O_Data = move_total - move_min          (counted in tensor elements, as the paper does)
    score  = w_mac * O_MAC + w_data * O_Data,   minimised over the candidates

This file holds the paper's arithmetic and nothing of any kernel: `select` takes every
candidate's issued MACs and moved elements as INPUTS.  For the rewrites the paper itself
describes, those two numbers follow from the paper and are computed here:

  MAC_min    = M*K*C*R*S, the MACs of the definition (M = N*P*Q output pixels).
  MAC_total  = MACs the matrix unit issues once every mapped dimension is padded to the
               unit's extent (x, y, z) (Sec. 4.2.4 rule b): ceil(M,x) * ceil(K,y) * depth,
               depth = fused reduction length of the candidate, padded to z.
  move_min   = |in| + |wt| + |out|.
  move_total = every element a layout rewrite reads or writes plus every element the
               GEMM stage reads or writes:
               (|in| + |X'|) + (|wt| + |W'|) + (|X'| + |W'| + |out|)
               with X' the rewritten input and W' the rewritten weights.

  blocked    channel blocks of cb (Pad + Split + Reorder, the reference mapping of Sec. 5.1):
             X' = N * ceil(C,cb) * (H+2p) * (W+2p), depth = ceil(ceil(C,cb)*R*S, z)
  unrolled   Stencil Unroll + Fuse (Table 2 rows 1 and 5): X' = M * depth, depth = ceil(C*R*S, z)
  image_packed  Image Pack (Table 2 row 1, strides above one) followed by a stride-1 candidate
             on the packed problem: that candidate's numbers, measured against the MACs of the
             ORIGINAL definition (the split kernel's zero taps are overhead), plus the pack's own
             traffic, which writes X2 and W2 for the inner stage to read again.

A candidate that the paper does not describe (anything a library adds) enters `select` with
numbers its author has to justify elsewhere; nothing about it is stated here.
"""
from __future__ import annotations

UNIT = (32, 32, 64)  # extents (x: pixels, y: output channels, z: depth) of the matrix unit checked


def _ceil(x, m):
    return -(-x // m) * m


def out_extent(N, C, H, W, K, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def mac_min(N, C, H, W, K, R, S, stride, pad):
    P, Q = out_extent(N, C, H, W, K, R, S, stride, pad)
    return N * P * Q * K * C * R * S


def move_min(N, C, H, W, K, R, S, stride, pad):
    P, Q = out_extent(N, C, H, W, K, R, S, stride, pad)
    return N * C * H * W + K * C * R * S + N * K * P * Q


def move_total(dims, x_elems, w_elems):
    """Rewrites read in, wt and write X', W'; the GEMM stage reads X', W' and writes out."""
    N, C, H, W, K, R, S, stride, pad = dims
    P, Q = out_extent(*dims)
    return (N * C * H * W + x_elems) + (K * C * R * S + w_elems) + (x_elems + w_elems + N * K * P * Q)


def overheads(dims, mac_total, moved):
    """(O_MAC, O_Data) of a candidate that issues `mac_total` MACs and moves `moved` elements."""
    return mac_total - mac_min(*dims), moved - move_min(*dims)


def score(o_mac, o_data, w_mac, w_data):
    return w_mac * o_mac + w_data * o_data


def blocked(dims, cb, unit=UNIT):
    """Channel blocks of cb: (MAC_total, move_total, rewritten elements)."""
    N, C, H, W, K, R, S, stride, pad = dims
    P, Q = out_extent(*dims)
    cpad = _ceil(C, cb)
    depth = _ceil(cpad * R * S, unit[2])
    x_elems = N * cpad * (H + 2 * pad) * (W + 2 * pad)
    w_elems = K * depth
    return _ceil(N * P * Q, unit[0]) * _ceil(K, unit[1]) * depth, move_total(dims, x_elems, w_elems), x_elems + w_elems


def unrolled(dims, unit=UNIT):
    """Stencil unroll + fuse: (MAC_total, move_total, rewritten elements)."""
    N, C, H, W, K, R, S, stride, pad = dims
    P, Q = out_extent(*dims)
    depth = _ceil(C * R * S, unit[2])
    x_elems = N * P * Q * depth
    w_elems = K * depth
    return _ceil(N * P * Q, unit[0]) * _ceil(K, unit[1]) * depth, move_total(dims, x_elems, w_elems), x_elems + w_elems


def image_pack_dims(N, C, H, W, K, R, S, stride, pad):
    """The stride-1, pad-0 problem whose channels are the stride phases (Table 2, Image Pack)."""
    P, Q = out_extent(N, C, H, W, K, R, S, stride, pad)
    R2, S2 = -(-R // stride), -(-S // stride)
    return (N, C * stride * stride, P + R2 - 1, Q + S2 - 1, K, R2, S2, 1, 0)


def image_packed(dims, inner_o_mac, inner_o_data, inner_rewritten):
    """(O_MAC, O_Data, rewritten) of Image Pack followed by a candidate on the packed problem
    whose own overheads (against the packed problem's definition) are given."""
    d2 = image_pack_dims(*dims)
    x2 = d2[0] * d2[1] * d2[2] * d2[3]
    w2 = d2[4] * d2[1] * d2[5] * d2[6]
    zero_taps = mac_min(*d2) - mac_min(*dims)
    return inner_o_mac + zero_taps, inner_o_data + 2 * (x2 + w2), inner_rewritten + x2 + w2


def select(cands, w_mac, w_data):
    """cands: iterable of (layout, cb, O_MAC, O_Data, rewritten).  Returns (layout, cb, score) of
    the cheapest.  Ties: fewer rewritten elements, then lower layout code, then larger block."""
    best = None
    for layout, cb, o_mac, o_data, rewritten in cands:
        sc = score(o_mac, o_data, w_mac, w_data)
        key = (sc, rewritten, layout, -cb)
        if best is None or key < best[0]:
            best = (key, layout, cb, sc)
    return best[1], best[2], best[3]
