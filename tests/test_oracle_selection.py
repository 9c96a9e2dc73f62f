"""Pins for the candidate-selection arithmetic (Sec. 4.4), CPU only.  Everything checked here is
fixed by the paper or by counting: the checker holds no kernel's geometry."""
import pytest

from oracle import selection as sel
from paper_2104_04731_amd.inputs import CONFIGS

PACKED, IM2COL, PAD_ONLY = 1, 2, 3
VTA = (1, 16, 16)   # the paper's GEMM core (Sec. 5.1)


def paper_candidates(dims, unit=sel.UNIT):
    """The rewrites the paper describes, with their overheads: channel blocks, one padded block, stencil unroll."""
    C = dims[1]
    out = []
    for layout, cb in [(PACKED, 64), (PACKED, 32), (PACKED, 16), (PAD_ONLY, -(-C // 16) * 16)]:
        mt, mv, rw = sel.blocked(dims, cb, unit)
        out.append((layout, cb, *sel.overheads(dims, mt, mv), rw))
    mt, mv, rw = sel.unrolled(dims, unit)
    out.append((IM2COL, 0, *sel.overheads(dims, mt, mv), rw))
    return out


def test_no_padding_means_no_mac_overhead():
    # every mapped dimension divides the unit: M = 2*16*16, K = 64, C = 64
    dims = (2, 64, 16, 16, 64, 1, 1, 1, 0)
    mt, mv, rw = sel.blocked(dims, 64)
    o_mac, o_data = sel.overheads(dims, mt, mv)
    assert o_mac == 0
    assert o_data == 2 * (2 * 64 * 16 * 16) + 2 * (64 * 64)     # X' and W' written once, read once
    assert rw == 2 * 64 * 16 * 16 + 64 * 64
    assert sel.overheads(dims, sel.mac_min(*dims), sel.move_min(*dims)) == (0, 0)


@pytest.mark.parametrize("C,cb", [(1, 16), (3, 16), (8, 16), (3, 64), (20, 32)])
def test_channel_padding_utilisation_law(C, cb):
    """Useful fraction of the issued MACs is ic / padded ic (Sec. 6.1); the inflation is at
    most the block size."""
    # R*S*cpad multiple of 64 and M, K multiples of 32 so that only channel padding counts
    N, H, W, K, R, S = 1, 32, 32, 32, 2, 2
    dims = (N, C, H + R - 1, W + S - 1, K, R, S, 1, 0)
    mac_total, _, _ = sel.blocked(dims, cb)
    mac_min = N * H * W * K * C * R * S
    assert sel.mac_min(*dims) == mac_min
    cpad = -(-C // cb) * cb
    assert mac_total * C == mac_min * cpad
    assert mac_total <= cb * mac_min


@pytest.mark.parametrize("ic", [1, 3, 5, 16, 17])
def test_utilisation_on_the_papers_own_unit(ic):
    """VTA's (1,16,16) core with z = 16 channel blocks: utilisation ic / ceil(ic,16), never worse than 1/16."""
    dims = (1, ic, 10, 10, 16, 3, 3, 1, 1)
    mac_total, _, _ = sel.blocked(dims, 16, VTA)
    assert mac_total * ic == sel.mac_min(*dims) * (-(-ic // 16) * 16)
    assert mac_total <= 16 * sel.mac_min(*dims)


def test_stencil_unroll_data_growth():
    # im2col writes M*depth elements: R*S-fold growth at stride 1 (Table 2 row 1: [N,I] -> [N,I,K])
    dims = (1, 64, 34, 34, 32, 3, 3, 1, 0)
    mt, mv, rw = sel.unrolled(dims)
    o_mac, o_data = sel.overheads(dims, mt, mv)
    assert o_mac == 0
    assert o_data == 2 * (32 * 32 * 576) + 2 * (32 * 576)
    assert rw == 32 * 32 * 576 + 32 * 576
    # the unrolled input alone is R*S times the pixels it covers
    assert 32 * 32 * 576 == 9 * (64 * 32 * 32)


def test_move_min_counts_each_tensor_once():
    dims = (2, 3, 5, 7, 4, 3, 2, 1, 0)      # P = 3, Q = 6
    assert sel.out_extent(*dims) == (3, 6)
    assert sel.move_min(*dims) == 2 * 3 * 5 * 7 + 4 * 3 * 3 * 2 + 2 * 4 * 3 * 6
    assert sel.move_total(dims, 0, 0) == sel.move_min(*dims)    # nothing rewritten, nothing moved twice
    assert sel.move_total(dims, 10, 1) == sel.move_min(*dims) + 2 * 10 + 2 * 1


def test_paper_weights_pick_unroll_for_low_channel_and_blocking_otherwise():
    """With w = [1,1] (Sec. 6) the MAC term dominates: one- and three-channel layers go to
    stencil unrolling, many-channel layers stay with channel blocking."""
    for name, want in [("C3", IM2COL), ("C5", IM2COL), ("C2", PACKED), ("C4a", PACKED), ("C4b", PACKED), ("C1", PACKED)]:
        layout, cb, score = sel.select(paper_candidates(CONFIGS[name].dims()), 1.0, 1.0)
        assert layout == want, name
        assert score >= 0
    assert sel.select(paper_candidates(CONFIGS["C2"].dims()), 1.0, 1.0)[1] == 64
    assert sel.select(paper_candidates(CONFIGS["C1"].dims()), 1.0, 1.0)[1] == 16


def test_weight_vector_shifts_the_choice():
    cands = paper_candidates(CONFIGS["C3"].dims())
    # a pure data-movement objective never picks the unrolled layout for a 7x7 stem
    assert sel.select(cands, 0.0, 1.0)[0] != IM2COL
    # a pure MAC objective does
    assert sel.select(cands, 1.0, 0.0)[0] == IM2COL


def test_score_is_the_weighted_sum_and_ties_are_deterministic():
    assert sel.score(3, 5, 2.0, 7.0) == 41.0
    cands = [(1, 16, 10, 10, 7), (1, 64, 10, 10, 7), (2, 0, 10, 10, 7), (3, 16, 10, 10, 9), (4, 0, 11, 10, 0)]
    assert sel.select(cands, 1.0, 1.0)[:2] == (1, 64)            # equal score and size: lower code, larger block
    assert sel.select(cands + [(5, 0, 10, 10, 6)], 1.0, 1.0)[:2] == (5, 0)   # fewer rewritten elements first
    assert sel.select(cands, 0.0, 1.0)[:2] == (4, 0)             # score ties at 10, nothing rewritten wins
    # C = 64: blocks of 16/32/64 and the single padded block describe equal-cost layouts
    layout, cb, _ = sel.select(paper_candidates((1, 64, 8, 8, 32, 3, 3, 1, 1)), 1.0, 1.0)
    assert (layout, cb) == (PACKED, 64)


def test_image_pack_candidate():
    """Image Pack exists for strides above one; its cost is the packed problem's plus the pack's own
    traffic, and the zero taps of the split kernel count as MAC overhead."""
    dims = (1, 4, 16, 16, 32, 2, 2, 2, 0)                     # 2x2 stride 2: no zero taps, P = Q = 8
    d2 = sel.image_pack_dims(*dims)
    assert d2 == (1, 16, 8, 8, 32, 1, 1, 1, 0)
    assert sel.mac_min(*d2) == sel.mac_min(*dims)
    imt, imv, irw = sel.blocked(d2, 16)
    io_mac, io_data = sel.overheads(d2, imt, imv)
    x2, w2 = 16 * 8 * 8, 32 * 16
    assert sel.image_packed(dims, io_mac, io_data, irw) == (io_mac, io_data + 2 * (x2 + w2), irw + x2 + w2)
    # 3x3 stride 2: the split kernel has 4 phases x 2x2 = 16 taps for 9 weights
    dims = (1, 16, 17, 17, 32, 3, 3, 2, 0)
    d2 = sel.image_pack_dims(*dims)
    assert d2 == (1, 64, 9, 9, 32, 2, 2, 1, 0)
    imt, imv, irw = sel.blocked(d2, 64)
    o_mac, _, _ = sel.image_packed(dims, *sel.overheads(d2, imt, imv), irw)
    assert o_mac == 64 * 32 * (64 * 4) - 64 * 32 * 16 * 9      # 64 pixels; depth 256 issued for 144 useful
    # strided low-channel layers (C3: 3 channels x 4 phases = 12, C5: 1 x 4 = 4): the phases fill the channel
    # block that padding alone fills with zeros, so Image Pack + blocks of 16 beats direct blocking on BOTH terms
    # (the paper's case for it, Sec. 6.1), while under w = [1,1] stencil unrolling still issues the fewest MACs
    for name in ("C3", "C5"):
        d = CONFIGS[name].dims()
        d2 = sel.image_pack_dims(*d)
        imt, imv, irw = sel.blocked(d2, 16)
        packed = sel.image_packed(d, *sel.overheads(d2, imt, imv), irw)
        mt, mv, rw = sel.blocked(d, 16)
        direct = sel.overheads(d, mt, mv)
        assert packed[0] < direct[0] and packed[1] < direct[1] and packed[2] < rw
        cands = paper_candidates(d) + [(5, 16, *packed)]
        assert sel.select(cands, 1.0, 1.0)[0] == IM2COL
        assert sel.select(cands, 0.0, 1.0)[:2] == (5, 16)       # smallest data movement of all
