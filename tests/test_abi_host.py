"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, validates arguments before touching the device, and its layout selector and size
queries agree with the independently written definitions."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import direct, layouts, selection as sel
from paper_2104_04731_amd.inputs import CONFIGS, PAPER_SHAPES

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "conv2d_int8.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|size_t|char)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_what_the_binding_lists(lib):
    assert declared_functions() == sorted(lib.EXPORTS)


def test_library_exports_every_declared_symbol(lib):
    raw = ctypes.CDLL(lib._build.LIB)
    for name in declared_functions():
        assert hasattr(raw, name), name


ALL_SHAPES = list(CONFIGS.values()) + PAPER_SHAPES


# The candidate list the header states for the selectors: (layout, block); PAD_ONLY's block is ceil(C,16).
def stated_candidates(C, stride):
    out = [(1, 64), (1, 32), (1, 16), (2, 0), (3, -(-C // 16) * 16), (4, 0)]
    if stride > 1:
        out += [(5, 0), (5, 64), (5, 32), (5, 16)]
    return out


def paper_overheads(dims, layout, cb):
    """(O_MAC, O_Data, rewritten) of the rewrites the paper describes, from the checker's own arithmetic."""
    if layout == 2:
        mt, mv, rw = sel.unrolled(dims)
    else:
        mt, mv, rw = sel.blocked(dims, cb)
    return (*sel.overheads(dims, mt, mv), rw)


def library_candidates(lib, dims):
    """Every stated candidate the library accepts for this problem, with the overheads it reports."""
    out = []
    for layout, cb in stated_candidates(dims[1], dims[7]):
        if lib.layout_applies(dims, layout, cb):
            out.append((layout, cb, *lib.layout_overheads(dims, layout, cb)))
    return out


@pytest.mark.parametrize("cfg", ALL_SHAPES, ids=lambda c: c.name)
def test_selector_matches_definition(lib, cfg):
    dims = cfg.dims()
    cands = library_candidates(lib, dims)
    # the paper's own rewrites always apply, and the library's numbers for them are the paper's arithmetic
    for layout, cb in stated_candidates(cfg.C, 1)[:5]:
        assert lib.layout_overheads(dims, layout, cb) == paper_overheads(dims, layout, cb)
    # Image Pack over channel blocks: the packed problem's terms against the original definition + the pack's traffic
    if cfg.stride > 1:
        d2 = sel.image_pack_dims(*dims)
        for cb in (16, 32, 64):
            assert lib.layout_overheads(dims, 5, cb) == sel.image_packed(dims, *paper_overheads(d2, 1, cb))
    # the selectors are the Sec. 4.4 minimisation over what the library itself reports per candidate
    for w in [(1.0, 1.0), (1.0, 0.0), (0.0, 1.0), (1.0 / 0.6e15, 1.0 / 4.0e12), (3.0, 7.0)]:
        got = lib.select_layout(dims, *w)
        want = sel.select(cands, *w)
        assert got[:2] == want[:2]
        assert got[2] == pytest.approx(want[2], rel=1e-12)


def test_default_selector_minimises_with_its_stated_weights(lib):
    for cfg in ALL_SHAPES:
        got = lib.select_layout(cfg.dims())
        cands = library_candidates(lib, cfg.dims())
        assert got[:2] in [c[:2] for c in cands]
        # no candidate scores lower under the library's weights (seconds per MAC / per byte, both positive)
        w = (1.0 / 0.6e15, 1.0 / 4.0e12)
        assert got[2] == pytest.approx(min(sel.score(c[2], c[3], *w) for c in cands), rel=1e-12)


def test_size_queries_match_definitions(lib):
    for cfg in ALL_SHAPES:
        N, C, H, W, K, R, S, st, pad = cfg.dims()
        for cb in (16, 32, 64):
            Cb = -(-C // cb)
            assert lib.pack_layout_bytes(N, C, H, W, cb, pad) == N * Cb * cb * (H + 2 * pad) * (W + 2 * pad)
            assert lib.pack_weights_depth(C, R, S, lib.LAYOUT_PACKED, cb) == layouts.packed_depth(C, R, S, cb)
        assert lib.pack_weights_depth(C, R, S, lib.LAYOUT_IM2COL, 0) == layouts.ceil_to(C * R * S, 64)
        assert lib.pack_weights_depth(C, R, S, lib.LAYOUT_PAD_ONLY, 0) == \
            layouts.packed_depth(C, R, S, layouts.ceil_to(C, 16))
        kg = layouts.ceil_to(C * R * S, 64)
        assert lib.im2col_bytes(N, C, H, W, R, S, st, pad, kg) == cfg.M * kg
        ws = lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_IM2COL, 0)
        assert ws >= cfg.M * kg + K * kg


def _null_call(lib, dims):
    """Invalid problems must be rejected before any pointer is used or any launch is made."""
    raw = lib.load()
    return raw.conv2d_int8(*dims, None, None, None, None)


@pytest.mark.parametrize("dims,want", [
    ((0, 1, 4, 4, 1, 3, 3, 1, 1), 1), ((1, 1, 4, 4, 1, 3, 3, 0, 1), 1), ((1, 1, 4, 4, 1, 3, 3, 1, -1), 1),
    ((1, 1, 2, 2, 1, 3, 3, 1, 0), 1), ((1, 1, 4, 4, 1, 7, 3, 1, 1), 1),
    ((1, 16384, 8, 8, 1, 3, 3, 1, 1), 3),          # C*R*S = 147456 > 131072
    ((1, 16, 8, 8, 4, 3, 3, 1, 1), 1),             # valid problem, null tensors
])
def test_validation_happens_before_device_work(lib, dims, want):
    assert _null_call(lib, dims) == want


def test_ex_and_packed_validation(lib):
    raw = lib.load()
    d = lib.ConvDesc(1, 16, 8, 8, 4, 3, 3, 1, 1)
    assert raw.conv2d_int8_packed(ctypes.byref(d), lib.LAYOUT_AUTO, 0, None, None, None, -1, 0, None) == 1
    assert raw.conv2d_int8_packed(ctypes.byref(d), lib.LAYOUT_PACKED, 24, None, None, None, -1, 0, None) == 2
    assert raw.conv2d_int8_packed(ctypes.byref(d), lib.LAYOUT_PACKED, 16, None, None, None, -1, 0, None) == 1
    assert raw.conv2d_int8_ex(ctypes.byref(d), 7, 0, None, None, 0, None, None, 0, None) == 1
    assert raw.pack_layout(1, 3, 4, 4, 5, 0, None, None, None) == 1      # null first
    assert raw.pack_layout_bytes(1, 3, 4, 4, 5, 0) == 0                    # cb not a multiple of 4
    assert raw.gemm_int8_nt(4, 4, 60, None, None, None, None) == 1
    assert raw.conv2d_int8_workspace_bytes(None, 0, 0, 0) == 0
    assert lib.status_string(3).startswith("reduction")
    assert lib.num_tiles() >= 4
    for t in range(lib.num_tiles()):
        r, c, th, steps = lib.tile_info(t)
        assert r % 32 == 0 and c % 32 == 0 and th % 64 == 0 and steps in (1, 2, 4)


@pytest.mark.parametrize("dims,layout,cb", [
    ((512, 8192, 14, 14, 4096, 3, 3, 1, 1), 1, 16), ((512, 8192, 14, 14, 4096, 3, 3, 1, 1), 1, 64),
    ((64, 2048, 267, 162, 1000, 20, 2, 2, 1), 0, 0), ((4, 14000, 9, 9, 512, 3, 3, 1, 1), 1, 64),
    ((2048, 4096, 7, 7, 2048, 3, 3, 1, 1), 2, 0)], ids=str)
def test_deep_reductions_get_a_tile_that_fits(lib, dims, layout, cb):
    """A deep reduction adds an offset per 16-byte chunk to the blocked layout's LDS footprint: the tile the
    library picks must be one it can launch (the picker and the launcher share one LDS figure), and a forced
    large ring whose footprint would not fit is refused as unsupported, not discovered at launch."""
    if layout == 0:
        layout, cb = lib.select_layout(dims)[:2]
    tile, split = lib.query_tiling(dims, layout, cb)
    assert tile >= 0 and split >= 1
    assert lib.tile_applies(dims, layout, cb, tile, split)
    assert 0 < lib.tile_lds_bytes(dims, layout, cb, tile, split) <= 160 * 1024
    table = 0 if layout == 2 else lib.pack_weights_depth(dims[1], dims[5], dims[6], layout, cb) // 4   # 16 B per 64-byte step
    refused = 0
    for t in range(lib.num_tiles()):
        need = lib.tile_lds_bytes(dims, layout, cb, t, 1)
        assert need <= 160 * 1024
        assert (need > 0) == lib.tile_applies(dims, layout, cb, t, 1)
        rows, cols, threads, steps = lib.tile_info(t)
        if need:
            assert need >= 2 * (rows + cols) * 64 * steps + table      # at least two ring stages + the offsets
        refused += need == 0
    if table > 16 * 1024:
        assert refused > 0     # the deepest rings do not fit beside an offset table of this size


IMPLICIT_DOMAIN = [(1, 1, 8, 3, 4, 3, 3, 1, 1), (1, 16, 64, 4000, 4, 4, 4, 40, 0), (1, 1, 64, 4000, 4, 4, 4, 40, 0),
                   (1, 16, 9, 9, 8, 4, 4, 1, 0), (1, 17, 9, 9, 8, 4, 4, 1, 0), (2, 3, 40, 40, 8, 3, 3, 2, 1),
                   (1, 4, 30, 70, 8, 5, 5, 3, 2), (1, 64, 8, 200, 8, 1, 1, 5, 0), (1, 2, 300, 9, 8, 30, 4, 1, 0),
                   (2, 64, 6, 6, 8, 1, 1, 1, 0), (2, 512, 14, 14, 128, 1, 1, 1, 0), (1, 576, 4, 4, 8, 1, 1, 1, 0),
                   (1, 128, 5, 5, 8, 1, 1, 1, 0), (1, 128, 6, 6, 8, 1, 1, 1, 1), (1, 32, 6, 6, 8, 1, 1, 1, 0)]


@pytest.mark.parametrize("dims", IMPLICIT_DOMAIN + [c.dims() for c in ALL_SHAPES], ids=str)
def test_gemm_stage_unroll_domain_and_sizes(lib, dims):
    """layout_overheads is the domain query for IMPLICIT: every other entry point accepts the layout exactly
    where it does.  Inside the domain nothing is rewritten (no workspace, O_Data = 0), and the MACs it reports
    are whole units of the matrix intrinsic, never fewer than stencil unrolling issues (any way of feeding the
    unit pads at least the three fused dimensions).  That the accepted shapes compute the right result is the
    GPU tests' business; that the reported MACs are the issued ones is checked against the hardware counter."""
    N, C, H, W, K, R, S, st, pad = dims
    ok = lib.layout_applies(dims, lib.LAYOUT_IMPLICIT)
    d = lib.ConvDesc(*dims)
    raw = lib.load()
    p = ctypes.c_void_p(256)
    # null tensors: INVALID_ARG where the layout applies (validated after the plan), UNSUPPORTED where it does not
    want = lib.ERR_INVALID_ARG if ok else lib.ERR_UNSUPPORTED
    assert raw.conv2d_int8_ex(ctypes.byref(d), lib.LAYOUT_IMPLICIT, 0, None, None, 0, None, None, 0, None) == want
    assert raw.conv2d_int8_packed(ctypes.byref(d), lib.LAYOUT_IMPLICIT, 0, None, None, None, -1, 0, None) == want
    assert raw.conv2d_int8_packed_requant(ctypes.byref(d), lib.LAYOUT_IMPLICIT, 0, None, p, p, 64, 0, 8, 1, None) == want
    t, s = ctypes.c_int(), ctypes.c_int()
    assert raw.conv2d_int8_query_tiling(ctypes.byref(d), lib.LAYOUT_IMPLICIT, 0, ctypes.byref(t), ctypes.byref(s)) == \
        (lib.OK if ok else lib.ERR_UNSUPPORTED)
    depth = lib.pack_weights_depth(C, R, S, lib.LAYOUT_IMPLICIT, 0)
    if ok:
        o_mac, o_data, rewritten = lib.layout_overheads(dims, lib.LAYOUT_IMPLICIT, 0)
        assert (o_data, rewritten) == (0, 0)
        issued = o_mac + sel.mac_min(*dims)
        assert issued % (32 * 32 * 64) == 0
        assert issued >= sel.unrolled(dims)[0]
        assert lib.conv2d_int8_workspace_bytes(dims, lib.LAYOUT_IMPLICIT, 0) == 0
        assert (t.value, s.value) == (-1, 1)
        assert not lib.tile_applies(dims, lib.LAYOUT_IMPLICIT, 0, 0, 1)
        # the stated weight order of pack_weights(IMPLICIT): rows of the checker's index map
        assert depth == layouts.pack_weights_implicit(np.zeros((2, C, R, S), np.int8)).shape[1]
    else:
        assert depth in (0, layouts.pack_weights_implicit(np.zeros((2, C, R, S), np.int8)).shape[1])


def test_gemm_stage_unroll_covers_the_low_channel_configurations(lib):
    """What the layout exists for (Sec. 6.2's data growth): the three- and one-channel configurations are inside
    its domain; the many-channel 3x3 layers are not asked of it."""
    for name in ("C1", "C3", "C5", "C4b"):
        assert lib.layout_applies(CONFIGS[name].dims(), lib.LAYOUT_IMPLICIT), name


@pytest.mark.parametrize("dims", [(1, 4, 16, 16, 32, 2, 2, 2, 0), (2, 3, 40, 40, 8, 7, 7, 2, 3), (1, 1, 41, 50, 32, 20, 5, 2, 0),
                                  (1, 16, 17, 17, 32, 3, 3, 3, 1), (1, 64, 9, 9, 8, 1, 1, 2, 0), (1, 2, 9, 9, 8, 3, 3, 1, 1)],
                         ids=str)
def test_image_pack_problem_and_sizes(lib, dims):
    N, C, H, W, K, R, S, st, pad = dims
    d = lib.ConvDesc(*dims)
    raw = lib.load()
    if st == 1:
        assert raw.image_pack_bytes(ctypes.byref(d)) == 0
        assert raw.image_pack_desc(ctypes.byref(d), ctypes.byref(lib.ConvDesc())) == lib.ERR_UNSUPPORTED
        assert lib.conv2d_int8_workspace_bytes(dims, lib.LAYOUT_IMAGE_PACK, 16) == 0
        return
    d2 = layouts.image_pack_dims(*dims)
    assert lib.image_pack_desc(dims) == d2 == sel.image_pack_dims(*dims)
    assert raw.image_pack_bytes(ctypes.byref(d)) == d2[0] * d2[1] * d2[2] * d2[3]
    assert raw.image_pack_weights_bytes(ctypes.byref(d)) == K * d2[1] * d2[5] * d2[6]
    for cb in (0, 16, 64):
        if cb == 0 and not lib.layout_applies(d2, lib.LAYOUT_IMPLICIT):
            assert not lib.layout_applies(dims, lib.LAYOUT_IMAGE_PACK, 0)
            continue
        inner_layout = lib.LAYOUT_IMPLICIT if cb == 0 else lib.LAYOUT_PACKED
        assert lib.layout_overheads(dims, lib.LAYOUT_IMAGE_PACK, cb) == \
            sel.image_packed(dims, *lib.layout_overheads(d2, inner_layout, cb))
        inner = lib.conv2d_int8_workspace_bytes(d2, inner_layout, cb)
        up = lambda v: -(-v // 256) * 256
        assert lib.conv2d_int8_workspace_bytes(dims, lib.LAYOUT_IMAGE_PACK, cb) == \
            up(d2[0] * d2[1] * d2[2] * d2[3]) + up(K * d2[1] * d2[5] * d2[6]) + inner
    # the GEMM-stage entry points take single-stage layouts only
    assert raw.conv2d_int8_packed(ctypes.byref(d), lib.LAYOUT_IMAGE_PACK, 16, None, None, None, -1, 0, None) != lib.OK
    assert lib.pack_weights_depth(C, R, S, lib.LAYOUT_IMAGE_PACK, 16) == 0


def test_validation_of_the_newer_entry_points(lib):
    """Every argument is checked before anything is enqueued: these calls pass null or bad arguments and
    must return a status without touching a device."""
    raw = lib.load()
    d = lib.ConvDesc(1, 3, 16, 16, 8, 3, 3, 2, 1)
    d2 = lib.ConvDesc()
    assert raw.pack_layout_nhwc(1, 3, 4, 4, 16, 0, None, None, None) == lib.ERR_INVALID_ARG
    assert raw.pack_layout_nhwc(1, 3, 4, 4, 8, 0, ctypes.c_void_p(256), ctypes.c_void_p(256), None) == lib.ERR_UNSUPPORTED
    assert raw.pack_layout_nhwc(1, 0, 4, 4, 16, 0, ctypes.c_void_p(256), ctypes.c_void_p(256), None) == lib.ERR_INVALID_ARG
    assert raw.image_pack_desc(ctypes.byref(d), None) == lib.ERR_INVALID_ARG
    assert raw.image_pack_desc(None, ctypes.byref(d2)) == lib.ERR_INVALID_ARG
    assert raw.image_pack_int8(ctypes.byref(d), None, None, None) == lib.ERR_INVALID_ARG
    assert raw.image_pack_int8(ctypes.byref(d), ctypes.c_void_p(256), ctypes.c_void_p(258), None) == lib.ERR_INVALID_ARG  # dst % 4
    assert raw.image_pack_weights(ctypes.byref(d), None, ctypes.c_void_p(256), None) == lib.ERR_INVALID_ARG
    assert raw.image_pack_bytes(None) == 0 and raw.image_pack_weights_bytes(None) == 0
    # IMAGE_PACK: only the two-stage entry points take it; a bad inner block is an invalid argument
    a = ctypes.c_int64()
    assert raw.layout_overheads(ctypes.byref(d), lib.LAYOUT_IMAGE_PACK, 24, ctypes.byref(a), None, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_ex(ctypes.byref(d), lib.LAYOUT_IMAGE_PACK, 16, None, None, 0, None, None, 0, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_ex(ctypes.byref(d), lib.LAYOUT_IMAGE_PACK, 16, ctypes.c_void_p(256), ctypes.c_void_p(256), 1,
                              ctypes.c_void_p(256), ctypes.c_void_p(256), 1 << 30, None) == lib.ERR_UNSUPPORTED   # packed weights
    assert raw.conv2d_int8_ex(ctypes.byref(d), lib.LAYOUT_IMAGE_PACK, 16, ctypes.c_void_p(256), ctypes.c_void_p(256), 0,
                              ctypes.c_void_p(256), ctypes.c_void_p(256), 16, None) == lib.ERR_WORKSPACE
    # IMPLICIT: forced tiles and splits, null operands
    d3 = lib.ConvDesc(1, 3, 16, 16, 8, 3, 3, 1, 1)
    assert raw.conv2d_int8_packed(ctypes.byref(d3), lib.LAYOUT_IMPLICIT, 0, None, None, None, -1, 0, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_packed(ctypes.byref(d3), lib.LAYOUT_IMPLICIT, 0, ctypes.c_void_p(256), ctypes.c_void_p(256),
                                  ctypes.c_void_p(256), 3, 1, None) == lib.ERR_UNSUPPORTED
    assert raw.conv2d_int8_ex(ctypes.byref(d3), lib.LAYOUT_IMPLICIT, 0, None, None, 0, None, None, 0, None) == lib.ERR_INVALID_ARG
    big = lib.ConvDesc(1, 256, 14, 14, 8, 3, 3, 1, 1)
    assert raw.conv2d_int8_ex(ctypes.byref(big), lib.LAYOUT_IMPLICIT, 0, ctypes.c_void_p(256), ctypes.c_void_p(256), 0,
                              ctypes.c_void_p(256), None, 0, None) == lib.ERR_UNSUPPORTED


# ---- dilated convolution: problem arithmetic and argument checks (no device work) ----------------
@pytest.mark.parametrize("case", [((1, 1, 7, 7, 1, 3, 3, 1, 0), 2), ((2, 3, 9, 10, 4, 3, 3, 1, 2), 2), ((1, 2, 11, 8, 3, 2, 3, 1, 3), 3),
                                  ((4, 64, 28, 28, 64, 3, 3, 1, 2), 2), ((1, 16, 33, 65, 8, 3, 3, 1, 4), 4)], ids=str)
def test_dilated_problem_and_sizes(lib, case):
    dims, d = case
    N, C, H, W, K, R, S, st, pad = dims
    raw = lib.load()
    desc = lib.ConvDesc(*dims)
    d2 = layouts.dilation_dims(N, C, H, W, K, R, S, pad, d)
    assert lib.dilated_desc(dims, d) == d2
    assert raw.dilation_pack_bytes(ctypes.byref(desc), d) == d2[0] * d2[1] * d2[2] * d2[3]
    P, Q = direct.out_hw_dilated(H, W, R, S, 1, pad, d)
    assert lib.dilated_out_hw(dims, d) == (P, Q)
    up = lambda v: -(-v // 256) * 256
    for layout, cb in ((lib.LAYOUT_PACKED, 16), (lib.LAYOUT_IM2COL, 0), (lib.LAYOUT_AUTO, 0)):
        il, icb = (layout, cb) if layout != lib.LAYOUT_AUTO else lib.select_layout(d2)[:2]
        inner = lib.conv2d_int8_workspace_bytes(d2, il, icb)
        o2 = d2[0] * K * (d2[2] - R + 1) * (d2[3] - S + 1) * 4
        # the sub-images' results are stored only when the dense problem runs in IMPLICIT
        assert lib.conv2d_int8_dilated_workspace_bytes(dims, d, layout, cb) == \
            up(d2[0] * d2[1] * d2[2] * d2[3]) + (up(o2) if il == lib.LAYOUT_IMPLICIT else 0) + inner


def test_dilated_validation(lib):
    raw = lib.load()
    ok = lib.ConvDesc(1, 3, 16, 16, 8, 3, 3, 1, 2)
    d2 = lib.ConvDesc()
    p = ctypes.c_void_p(256)
    assert raw.dilated_desc(ctypes.byref(ok), 2, ctypes.byref(d2)) == lib.OK
    assert raw.dilated_desc(ctypes.byref(ok), 2, None) == lib.ERR_INVALID_ARG
    assert raw.dilated_desc(None, 2, ctypes.byref(d2)) == lib.ERR_INVALID_ARG
    assert raw.dilated_desc(ctypes.byref(ok), 0, ctypes.byref(d2)) == lib.ERR_INVALID_ARG
    assert raw.dilated_desc(ctypes.byref(ok), 1, ctypes.byref(d2)) == lib.ERR_UNSUPPORTED      # nothing to pack
    assert raw.dilated_desc(ctypes.byref(ok), 65, ctypes.byref(d2)) == lib.ERR_INVALID_ARG     # spread kernel 129 > 20
    assert raw.dilated_desc(ctypes.byref(lib.ConvDesc(1, 3, 200, 200, 8, 2, 2, 1, 0)), 65, ctypes.byref(d2)) == lib.ERR_UNSUPPORTED
    assert raw.dilated_desc(ctypes.byref(lib.ConvDesc(1, 3, 16, 16, 8, 3, 3, 2, 2)), 2, ctypes.byref(d2)) == lib.ERR_UNSUPPORTED  # stride
    assert raw.dilated_desc(ctypes.byref(lib.ConvDesc(1, 3, 4, 4, 8, 3, 3, 1, 0)), 2, ctypes.byref(d2)) == lib.ERR_INVALID_ARG   # extent 5 > 4
    assert raw.dilation_pack_bytes(None, 2) == 0 and raw.dilation_pack_bytes(ctypes.byref(ok), 1) == 0
    assert raw.dilation_pack_int8(ctypes.byref(ok), 2, None, p, None) == lib.ERR_INVALID_ARG
    assert raw.dilation_pack_int8(ctypes.byref(ok), 2, p, None, None) == lib.ERR_INVALID_ARG
    assert raw.dilation_unpack_int32(ctypes.byref(ok), 2, None, p, None) == lib.ERR_INVALID_ARG
    assert raw.dilation_unpack_int32(ctypes.byref(ok), 1, p, p, None) == lib.ERR_UNSUPPORTED
    assert raw.conv2d_int8_dilated_workspace_bytes(ctypes.byref(ok), 2, 99, 0) == 0
    assert raw.conv2d_int8_dilated_workspace_bytes(ctypes.byref(ok), 1, lib.LAYOUT_PACKED, 16) == 0
    need = raw.conv2d_int8_dilated_workspace_bytes(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 16)
    assert need > 0
    assert raw.conv2d_int8_dilated(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 16, None, p, p, p, need, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_dilated(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 16, p, p, p, None, need, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_dilated(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 16, p, p, p, ctypes.c_void_p(264), need, None) == lib.ERR_INVALID_ARG
    assert raw.conv2d_int8_dilated(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 16, p, p, p, p, need - 1, None) == lib.ERR_WORKSPACE
    assert raw.conv2d_int8_dilated(ctypes.byref(ok), 2, lib.LAYOUT_PACKED, 24, p, p, p, p, need, None) == lib.ERR_UNSUPPORTED


def test_fused_activation_validation(lib):
    raw = lib.load()
    d = lib.ConvDesc(1, 64, 14, 14, 128, 3, 3, 1, 1)
    p = ctypes.c_void_p(256)
    call = lambda layout=lib.LAYOUT_PACKED, cb=64, x=p, w=p, o=p, ocb=64, opad=0, shift=8, relu=1: \
        raw.conv2d_int8_packed_requant(ctypes.byref(d), layout, cb, x, w, o, ocb, opad, shift, relu, None)
    assert call(layout=lib.LAYOUT_AUTO) == lib.ERR_INVALID_ARG
    assert call(x=None) == lib.ERR_INVALID_ARG and call(w=None) == lib.ERR_INVALID_ARG and call(o=None) == lib.ERR_INVALID_ARG
    assert call(o=ctypes.c_void_p(260)) == lib.ERR_INVALID_ARG
    assert call(shift=32) == lib.ERR_INVALID_ARG and call(shift=-1) == lib.ERR_INVALID_ARG and call(opad=-1) == lib.ERR_INVALID_ARG
    assert call(ocb=24) == lib.ERR_UNSUPPORTED and call(ocb=128) == lib.ERR_UNSUPPORTED
    assert call(cb=24) == lib.ERR_UNSUPPORTED
    d1 = lib.ConvDesc(1, 64, 14, 14, 128, 3, 3, 1, 1)   # outside IMPLICIT's domain
    assert raw.conv2d_int8_packed_requant(ctypes.byref(d1), lib.LAYOUT_IMPLICIT, 0, p, p, p, 64, 0, 8, 1, None) == lib.ERR_UNSUPPORTED


def test_direct_dilated_validation(lib):
    raw = lib.load()
    ok = lib.ConvDesc(1, 3, 16, 16, 8, 3, 3, 2, 2)
    p = ctypes.c_void_p(256)
    need = raw.conv2d_int8_dilated_direct_workspace_bytes(ctypes.byref(ok), 2, 16)
    assert need == lib.conv2d_int8_workspace_bytes((1, 3, 16, 16, 8, 3, 3, 2, 2), lib.LAYOUT_PACKED, 16)
    assert raw.conv2d_int8_dilated_direct_workspace_bytes(ctypes.byref(ok), 0, 16) == 0
    assert raw.conv2d_int8_dilated_direct_workspace_bytes(ctypes.byref(ok), 10, 16) == 0    # spread extent 21 > 20
    assert raw.conv2d_int8_dilated_direct_workspace_bytes(None, 2, 16) == 0
    call = lambda dil=2, cb=16, x=p, w=p, o=p, ws=p, nb=need: raw.conv2d_int8_dilated_direct(ctypes.byref(ok), dil, cb, x, w, o, ws, nb, None)
    assert call(dil=0) == lib.ERR_INVALID_ARG and call(dil=10) == lib.ERR_INVALID_ARG
    assert call(x=None) == lib.ERR_INVALID_ARG and call(ws=None) == lib.ERR_INVALID_ARG
    assert call(ws=ctypes.c_void_p(264)) == lib.ERR_INVALID_ARG
    assert call(nb=need - 1) == lib.ERR_WORKSPACE
    assert call(cb=24) == lib.ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: any other count ends with a message and a non-zero status before anything is imported."""
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0 and "one GPU only" in r.stderr and r.stdout.strip() == ""


def test_im2col_nhwc_validation(lib):
    raw = lib.load()
    p = ctypes.c_void_p(256)
    assert raw.im2col_nhwc_int8(1, 3, 8, 8, 3, 3, 1, 1, 64, None, p, None) == lib.ERR_INVALID_ARG
    assert raw.im2col_nhwc_int8(1, 3, 8, 8, 3, 3, 1, 1, 64, p, ctypes.c_void_p(260), None) == lib.ERR_INVALID_ARG
    assert raw.im2col_nhwc_int8(1, 16, 8, 8, 3, 3, 1, 1, 192, ctypes.c_void_p(260), p, None) == lib.ERR_INVALID_ARG  # 16-byte loads
    assert raw.im2col_nhwc_int8(1, 3, 8, 8, 3, 3, 1, 1, 16, p, p, None) == lib.ERR_INVALID_ARG   # kg_pad < 27
    assert raw.im2col_nhwc_int8(1, 3, 8, 8, 3, 3, 1, 1, 40, p, p, None) == lib.ERR_INVALID_ARG   # not a multiple of 16
    assert raw.im2col_nhwc_int8(1, 3, 2, 2, 5, 5, 1, 0, 128, p, p, None) == lib.ERR_INVALID_ARG  # kernel larger than the image
    assert raw.pack_weights_rsc(0, 3, 3, 3, p, p, None) == lib.ERR_INVALID_ARG
    assert raw.pack_weights_rsc(4, 3, 3, 3, None, p, None) == lib.ERR_INVALID_ARG
    assert raw.pack_weights_rsc(4, 65536, 3, 3, p, p, None) == lib.ERR_OVERFLOW_RISK
