"""Pins for the candidate-selection overheads (Sec. 4.4), CPU only."""
import pytest

from oracle import selection as sel
from paper_2104_04731_amd.inputs import CONFIGS


def test_no_padding_means_no_mac_overhead():
    # every mapped dimension divides the unit: M=N*P*Q=64*..., K=64, C=64
    o_mac, o_data, _ = sel.overheads(2, 64, 16, 16, 64, 1, 1, 1, 0, sel.PACKED, 64)
    assert o_mac == 0
    assert o_data == 2 * (2 * 64 * 16 * 16) + 2 * (64 * 64)


@pytest.mark.parametrize("C,cb", [(1, 16), (3, 16), (8, 16), (3, 64), (20, 32)])
def test_channel_padding_utilisation_law(C, cb):
    """Useful fraction of the issued MACs is ic / padded ic (Sec. 6.1); the inflation is at
    most the block size."""
    # R*S*cpad multiple of 64 and M, K multiples of 32 so that only channel padding counts
    N, H, W, K, R, S = 1, 32, 32, 32, 2, 2
    o_mac, _, _ = sel.overheads(N, C, H + R - 1, W + S - 1, K, R, S, 1, 0, sel.PACKED, cb)
    mac_min = N * H * W * K * C * R * S
    cpad = -(-C // cb) * cb
    assert (o_mac + mac_min) * C == mac_min * cpad
    assert (o_mac + mac_min) <= cb * mac_min


def test_stencil_unroll_data_growth():
    # im2col writes M*depth elements: R*S-fold growth at stride 1 (Table 2 row 1: [N,I] -> [N,I,K])
    N, C, H, W, K, R, S = 1, 64, 34, 34, 32, 3, 3
    _, o_data, _ = sel.overheads(N, C, H, W, K, R, S, 1, 0, sel.IM2COL, 0)
    assert o_data == 2 * (32 * 32 * 576) + 2 * (32 * 576)


def test_paper_weights_pick_unroll_for_low_channel_and_blocking_otherwise():
    """With w = [1,1] (Sec. 6) the MAC term dominates: one- and three-channel layers go to
    stencil unrolling, many-channel layers stay with channel blocking."""
    for name, want in [("C3", sel.IM2COL), ("C5", sel.IM2COL), ("C2", sel.PACKED),
                       ("C4a", sel.PACKED), ("C4b", sel.PACKED), ("C1", sel.PACKED)]:
        layout, cb, score = sel.select(*CONFIGS[name].dims(), 1.0, 1.0)
        assert layout == want, name
        assert score >= 0
    assert sel.select(*CONFIGS["C2"].dims(), 1.0, 1.0)[1] == 64
    assert sel.select(*CONFIGS["C1"].dims(), 1.0, 1.0)[1] == 16


def test_weight_vector_shifts_the_choice():
    # a pure data-movement objective never picks the unrolled layout for a 7x7 stem
    layout, cb, _ = sel.select(*CONFIGS["C3"].dims(), 0.0, 1.0)
    assert layout != sel.IM2COL
    # a pure MAC objective does
    assert sel.select(*CONFIGS["C3"].dims(), 1.0, 0.0)[0] == sel.IM2COL


def test_tie_breaks_are_deterministic():
    # C=64: blocks of 16/32/64 and the single padded block describe equal-cost layouts
    layout, cb, _ = sel.select(1, 64, 8, 8, 32, 3, 3, 1, 1, 1.0, 1.0)
    assert (layout, cb) == (sel.PACKED, 64)


def test_unrolling_inside_the_gemm_stage_moves_nothing_twice():
    """Its only overhead is the matrix unit's padding: kernel rows to four taps, the depth to 64,
    each output row to 32 pixels, output channels to 32."""
    N, C, H, W, K, R, S = 2, 2, 10, 35, 32, 4, 4           # P=7, Q=32: nothing to pad but the depth
    o_mac, o_data, rewritten = sel.overheads(N, C, H, W, K, R, S, 1, 0, sel.IMPLICIT, 0)
    assert (o_data, rewritten) == (0, 0)
    assert o_mac == N * 7 * 32 * K * (64 - C * R * S)
    # 7-tap rows are issued as 8: useful fraction 7/8 when everything else divides
    o_mac, _, _ = sel.overheads(1, 8, 8, 38, 32, 1, 7, 1, 0, sel.IMPLICIT, 0)   # Q=32, depth 8*1*8=64
    mac_min = 8 * 32 * 32 * 8 * 7
    assert (o_mac + mac_min) * 7 == mac_min * 8


def test_domain_of_unrolling_inside_the_gemm_stage():
    assert sel.implicit_applies(*CONFIGS["C3"].dims()) and sel.implicit_applies(*CONFIGS["C5"].dims())
    assert sel.implicit_applies(*CONFIGS["C1"].dims())                       # 16*3*4 = 192 deep
    for name in ("C2", "C4a"):                                                # 768, 3072 deep
        assert not sel.implicit_applies(*CONFIGS[name].dims())
        assert (sel.IMPLICIT, 0) not in sel.candidates(CONFIGS[name].C, CONFIGS[name].dims())
    assert sel.implicit_applies(*CONFIGS["C4b"].dims())                      # 1x1 form: depth = C = 512
    assert not sel.implicit_applies(1, 1, 8, 3, 4, 3, 3, 1, 1)                # three-pixel rows
    assert not sel.implicit_applies(1, 16, 64, 4000, 4, 4, 4, 40, 0)          # 16 channels x 4 rows x 5 KB
    assert sel.implicit_applies(1, 1, 64, 4000, 4, 4, 4, 40, 0)


def test_hardware_weights_send_low_channel_layers_to_the_gemm_stage_unroll():
    """With seconds per MAC and per moved byte as weights, writing and re-reading the unrolled matrix
    costs far more than the padded MACs: C3 and C5 leave im2col; the paper's w = [1,1] keeps it."""
    for name in ("C3", "C5"):
        assert sel.select(*CONFIGS[name].dims(), 1.0 / 0.6e15, 1.0 / 4.0e12)[0] == sel.IMPLICIT
        assert sel.select(*CONFIGS[name].dims(), 1.0, 1.0)[0] == sel.IM2COL


def test_pointwise_form_of_the_gemm_stage_unroll():
    """1x1 over whole 64-channel multiples: no kernel-row padding, pixels padded per image."""
    N, C, H, W, K = 8, 512, 14, 14, 128
    o_mac, o_data, rewritten = sel.overheads(N, C, H, W, K, 1, 1, 1, 0, sel.IMPLICIT, 0)
    assert (o_data, rewritten) == (0, 0)
    assert o_mac == N * (224 - 196) * K * C                        # 196 pixels issued as 7 x 32
    assert sel.overheads(2, 64, 8, 8, 32, 1, 1, 1, 0, sel.IMPLICIT, 0)[0] == 0
    for dims in [(1, 128, 6, 6, 8, 1, 1, 2, 0), (1, 128, 6, 6, 8, 1, 1, 1, 1), (1, 576, 4, 4, 8, 1, 1, 1, 0),
                 (1, 128, 5, 5, 8, 1, 1, 1, 0)]:                   # stride, padding, depth, pixel count
        assert not sel.implicit_applies(*dims)
    # the hardware weights prefer it to channel blocking (nothing moved twice); w = [1,1] does not
    assert sel.select(*CONFIGS["C4b"].dims(), 1.0 / 0.6e15, 1.0 / 4.0e12)[0] == sel.IMPLICIT
    assert sel.select(*CONFIGS["C4b"].dims(), 1.0, 1.0)[0] == sel.PACKED


def test_image_pack_candidate():
    """Image Pack exists for strides above one; its cost is the packed problem's plus the pack's own
    traffic; on a unit that strides for free it never beats the direct layouts of these shapes."""
    dims = (1, 4, 16, 16, 32, 2, 2, 2, 0)                     # 2x2 stride 2: no zero taps, P = Q = 8
    assert sel.image_pack_dims(*dims) == (1, 16, 8, 8, 32, 1, 1, 1, 0)
    o_mac, o_data, rewritten = sel.overheads(*dims, sel.IMAGE_PACK, 16)
    x2, w2 = 16 * 8 * 8, 32 * 16
    inner = sel.overheads(1, 16, 8, 8, 32, 1, 1, 1, 0, sel.PACKED, 16)
    assert (o_mac, o_data, rewritten) == (inner[0], inner[1] + 2 * (x2 + w2), inner[2] + x2 + w2)
    # 3x3 stride 2: the split kernel has 4x4 = 16 taps for 9 weights
    dims = (1, 16, 17, 17, 32, 3, 3, 2, 0)
    d2 = sel.image_pack_dims(*dims)
    assert d2 == (1, 64, 9, 9, 32, 2, 2, 1, 0)
    o_mac, _, _ = sel.overheads(*dims, sel.IMAGE_PACK, 64)
    assert o_mac == 64 * 32 * (64 * 4) - 64 * 32 * 16 * 9      # 64 pixels; depth 256 issued for 144 useful
    assert all(lay != sel.IMAGE_PACK for lay, _ in sel.candidates(16, (1, 16, 17, 17, 32, 3, 3, 1, 0)))
    for name in ("C3", "C5"):
        for w in ((1.0, 1.0), (1.0 / 0.6e15, 1.0 / 4.0e12), (0.0, 1.0), (1.0, 0.0)):
            assert sel.select(*CONFIGS[name].dims(), *w)[0] != sel.IMAGE_PACK
