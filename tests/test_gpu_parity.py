"""GPU parity: every kernel, through the C-ABI, against the CPU definitions, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import direct, layouts
from paper_2104_04731_amd.inputs import CONFIGS, PAPER_SHAPES, ConvShape, uniform_int8

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


_ORACLE_CACHE = {}


def oracle_conv(cfg):
    if cfg.name not in _ORACLE_CACHE:
        x, w = cfg.make()
        _ORACLE_CACHE[cfg.name] = (x, w, direct.conv2d_int8(x, w, cfg.stride, cfg.pad))
    return _ORACLE_CACHE[cfg.name]


# ---- layout rewrites ----------------------------------------------------------------------
@pytest.mark.parametrize("shape,cb,pad", [
    ((600, 200, 7, 9), 64, 2), ((1100, 64, 12, 16), 64, 1), ((90, 130, 20, 23), 128, 3), ((4100, 64, 3, 5), 64, 0),
    ((520, 70, 14, 14), 64, 1),
])
def test_pack_layout_destination_order(lib, shape, cb, pad):
    """Enough 64-record units to fill the chip: the kernel then works in destination order (whole-line stores with
    the border inside them).  Planes whose size is not a multiple of four take that form at any size, so the small
    shapes above cover its edge cases too; these cover its index arithmetic over many planes."""
    N, C, H, W = shape
    assert N * -(-C // cb) * (cb // 64) * -(-(H + 2 * pad) * (W + 2 * pad) // 64) >= 4096
    x = uniform_int8(sum(shape) + cb + pad, shape)
    got = host(lib.pack_layout(dev(x), cb, pad))
    np.testing.assert_array_equal(got, layouts.pack_layout(x, cb, pad))


@pytest.mark.parametrize("shape,cb,pad", [
    ((2, 37, 5, 6), 16, 1), ((1, 3, 31, 29), 16, 3), ((3, 64, 14, 14), 64, 1), ((1, 70, 9, 130), 32, 0),
    ((1, 16, 14, 14), 16, 1), ((2, 5, 7, 7), 4, 2), ((2, 20, 7, 9), 8, 1), ((1, 1, 161, 500), 16, 0),
    ((1, 100, 3, 3), 112, 2), ((1, 1, 1, 1), 16, 0),
])
def test_pack_layout(lib, shape, cb, pad):
    x = uniform_int8(sum(shape) + cb, shape)
    got = host(lib.pack_layout(dev(x), cb, pad))
    np.testing.assert_array_equal(got, layouts.pack_layout(x, cb, pad))


@pytest.mark.parametrize("shape,cb,pad", [
    ((2, 70, 6, 10), 64, 2), ((1, 130, 14, 14), 128, 1), ((3, 64, 8, 8), 64, 0), ((1, 64, 5, 4), 64, 3),
    ((2, 200, 9, 12), 64, 1), ((1, 64, 56, 56), 64, 1), ((2, 64, 1, 4), 64, 1), ((1, 65, 16, 20), 192, 1),
])
def test_pack_layout_64_channel_slices(lib, shape, cb, pad):
    """Shapes the wave-tiled kernel takes: partial last chunk, dead channels, several slices per block,
    row ends inside a chunk, top and bottom border rows wider than a chunk."""
    x = uniform_int8(sum(shape) + cb + pad, shape)
    got = host(lib.pack_layout(dev(x), cb, pad))
    np.testing.assert_array_equal(got, layouts.pack_layout(x, cb, pad))


@pytest.mark.parametrize("shape,cb,pad", [
    ((2, 37, 5, 6), 16, 1), ((1, 3, 31, 29), 16, 3), ((3, 64, 14, 14), 64, 1), ((1, 70, 9, 130), 32, 0),
    ((1, 256, 14, 14), 64, 1), ((2, 20, 7, 9), 48, 2), ((1, 1, 16, 50), 16, 0), ((1, 130, 3, 3), 128, 1),
])
def test_pack_layout_nhwc_source(lib, shape, cb, pad):
    """Channel blocking from an NHWC source: same destination as from NCHW, for whole and ragged channel
    counts (16-byte pieces, byte tails, dead channels) and at an odd source alignment."""
    x = uniform_int8(sum(shape) + cb, shape)                      # NCHW values ...
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))             # ... stored NHWC
    want = layouts.pack_layout_nhwc(xh, cb, pad)
    np.testing.assert_array_equal(host(lib.pack_layout_nhwc(dev(xh), cb, pad)), want)
    np.testing.assert_array_equal(want, layouts.pack_layout(x, cb, pad))
    buf = torch.zeros(xh.size + 8, dtype=torch.int8, device=DEV)
    dx = buf[3:3 + xh.size].view(xh.shape); dx.copy_(dev(xh))
    np.testing.assert_array_equal(host(lib.pack_layout_nhwc(dx, cb, pad)), want)


@pytest.mark.parametrize("name", ["C2", "C3", "C4a", "C5"])
def test_pack_layout_configs(lib, name):
    cfg = CONFIGS[name]
    x, _ = cfg.make()
    for cb in (16, 64):
        np.testing.assert_array_equal(host(lib.pack_layout(dev(x), cb, cfg.pad)),
                                      layouts.pack_layout(x, cb, cfg.pad))


@pytest.mark.parametrize("wshape,cb", [((5, 3, 7, 7), 16), ((16, 16, 3, 3), 16), ((7, 40, 3, 2), 32),
                                       ((64, 64, 3, 3), 64), ((9, 70, 1, 1), 64), ((3, 33, 2, 3), 48),
                                       ((32, 1, 20, 5), 16)])
def test_pack_weights(lib, wshape, cb):
    w = uniform_int8(sum(wshape), wshape)
    got = host(lib.pack_weights(dev(w), lib.LAYOUT_PACKED, cb))
    np.testing.assert_array_equal(got, layouts.pack_weights_blocked(w, cb))
    got = host(lib.pack_weights(dev(w), lib.LAYOUT_IM2COL, 0))
    np.testing.assert_array_equal(got, layouts.pack_weights_im2col(w))
    cbp = layouts.ceil_to(wshape[1], 16)
    if layouts.ceil_to(w.shape[1] * w.shape[2] * layouts.ceil_to(w.shape[3], 4), 64) <= 256:
        got = host(lib.pack_weights(dev(w), lib.LAYOUT_IMPLICIT, 0))
        np.testing.assert_array_equal(got, layouts.pack_weights_implicit(w))
    else:
        with pytest.raises(lib.ConvError) as e:
            lib.pack_weights(dev(w), lib.LAYOUT_IMPLICIT, 0)
        assert e.value.status == lib.ERR_UNSUPPORTED
    got = host(lib.pack_weights(dev(w), lib.LAYOUT_PAD_ONLY, 0))
    np.testing.assert_array_equal(got, layouts.pack_weights_blocked(w, cbp))


@pytest.mark.parametrize("dims", [(2, 3, 6, 7, 3, 2, 2, 1), (1, 3, 31, 29, 7, 7, 2, 3), (1, 16, 14, 14, 3, 3, 1, 1),
                                  (2, 1, 41, 50, 20, 5, 2, 0), (1, 5, 9, 9, 1, 1, 1, 0), (1, 2, 5, 5, 7, 7, 1, 1),
                                  (1, 70, 6, 6, 3, 3, 3, 2)])
def test_im2col(lib, dims):
    N, C, H, W, R, S, st, pad = dims
    x = uniform_int8(sum(dims), (N, C, H, W))
    got = host(lib.im2col_int8(dev(x), R, S, st, pad))
    np.testing.assert_array_equal(got, layouts.im2col(x, R, S, st, pad))


def test_im2col_random_shapes(lib):
    """Seeded random shapes over the unroll kernel's paths: wide and narrow rows, strides 1-3, kernel rows shorter
    and longer than a dword, pads up to the kernel size, channel counts that need several slices, tile tails."""
    rng = np.random.default_rng(20260)
    done = 0
    while done < 48:
        S = int(rng.integers(1, 8)); R = int(rng.integers(1, 6))
        st = int(rng.integers(1, 4)); pad = int(rng.integers(0, max(R, S) + 1))
        W = int(rng.integers(max(4, S), 90)); H = int(rng.integers(R, 24))
        C = int(rng.choice([1, 2, 3, 5, 16, 40, 130, 300])); N = int(rng.integers(1, 4))
        if (H + 2 * pad - R) // st + 1 < 1 or (W + 2 * pad - S) // st + 1 < 1 or N * C * H * W > 400000:
            continue
        x = uniform_int8(1000 + done, (N, C, H, W))
        got = host(lib.im2col_int8(dev(x), R, S, st, pad))
        np.testing.assert_array_equal(got, layouts.im2col(x, R, S, st, pad), err_msg=str((N, C, H, W, R, S, st, pad)))
        done += 1


@pytest.mark.parametrize("name", ["C3", "C5"])
def test_im2col_configs(lib, name):
    cfg = CONFIGS[name]
    x, _ = cfg.make()
    got = host(lib.im2col_int8(dev(x), cfg.R, cfg.S, cfg.stride, cfg.pad))
    np.testing.assert_array_equal(got, layouts.im2col(x, cfg.R, cfg.S, cfg.stride, cfg.pad))


# ---- the matrix intrinsic -------------------------------------------------------------------
def test_gemm_unit_hand_example(lib):
    A = np.zeros((1, 64), np.int8); A[0, :16] = np.arange(1, 17)
    B = np.zeros((16, 64), np.int8)
    B[:, :16] = np.array([[y - z for z in range(16)] for y in range(16)])
    got = host(lib.gemm_int8_nt(dev(A), dev(B)))
    np.testing.assert_array_equal(got[0], 136 * np.arange(16) - 1360)


@pytest.mark.parametrize("X,Y,Z", [(1, 1, 64), (33, 65, 128), (70, 300, 192), (129, 257, 64), (300, 130, 640),
                                   (16, 196, 192), (512, 100, 2304)])
def test_gemm_nt(lib, X, Y, Z):
    A = uniform_int8(X * 7 + Z, (X, Z)); B = uniform_int8(Y * 3 + Z, (Y, Z))
    np.testing.assert_array_equal(host(lib.gemm_int8_nt(dev(A), dev(B))), layouts.gemm_nt(A, B))


def test_gemm_every_tile_and_split(lib):
    """Each tile shape, with and without a depth split, on a ragged problem spanning several tiles."""
    for Z, splits in ((512, (1, 2, 4)), (448, (1, 2, 3, 7))):  # 8 and 7 depth steps
        X, Y = 300, 530
        cfg = ConvShape("g", 1, Z, 1, Y, X, 1, 1, 1, 0)
        A = uniform_int8(901 + Z, (X, Z)); B = uniform_int8(902 + Z, (Y, Z))
        want = layouts.gemm_nt(A, B).reshape(1, X, 1, Y)
        dA, dB = dev(A), dev(B)
        for tile in range(lib.num_tiles()):
            steps = lib.tile_info(tile)[3]
            for split in splits:
                out = torch.full((1, X, 1, Y), -7, dtype=torch.int32, device=DEV)
                per = -(-(Z // 64) // split)
                rule = (Z // 64) % steps == 0 and per % steps == 0   # whole stages per slice
                runnable = lib.tile_applies(cfg.dims(), lib.LAYOUT_IM2COL, 0, tile, split)
                assert runnable == rule
                # a row-major [Y][Z] matrix is the im2col operand of a 1x1 convolution over Y pixels
                if not runnable:
                    with pytest.raises(lib.ConvError) as e:
                        lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_IM2COL, 0, dB, dA, out, tile=tile, split_k=split)
                    assert e.value.status == lib.ERR_UNSUPPORTED
                    continue
                lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_IM2COL, 0, dB, dA, out, tile=tile, split_k=split)
                np.testing.assert_array_equal(host(out), want, err_msg=f"tile {tile} split {split} Z {Z}")


# ---- convolution ----------------------------------------------------------------------------
LAYOUT_CASES = [("packed", 16), ("packed", 32), ("packed", 64), ("im2col", 0), ("pad_only", 0)]


def run_layout(lib, cfg, x, w, lname, cb, tile=-1, split_k=0):
    lay = {"packed": lib.LAYOUT_PACKED, "im2col": lib.LAYOUT_IM2COL, "pad_only": lib.LAYOUT_PAD_ONLY}[lname]
    dx, dw = dev(x), dev(w)
    if lay == lib.LAYOUT_IM2COL:
        xp = lib.im2col_int8(dx, cfg.R, cfg.S, cfg.stride, cfg.pad)
    else:
        cbe = cb if lay == lib.LAYOUT_PACKED else layouts.ceil_to(cfg.C, 16)
        xp = lib.pack_layout(dx, cbe, cfg.pad)
    wp = lib.pack_weights(dw, lay, cb)
    out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), 12345, dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(cfg.dims(), lay, cb, xp, wp, out, tile=tile, split_k=split_k)
    return host(out)


@pytest.mark.parametrize("name", list(CONFIGS))
@pytest.mark.parametrize("lname,cb", LAYOUT_CASES)
def test_conv_configs_every_layout(lib, name, lname, cb):
    cfg = CONFIGS[name]
    x, w, want = oracle_conv(cfg)
    got = run_layout(lib, cfg, x, w, lname, cb)
    assert np.array_equal(got, want), f"{name} {lname} cb={cb}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("name", list(CONFIGS))
def test_conv_configs_one_shot(lib, name):
    cfg = CONFIGS[name]
    x, w, want = oracle_conv(cfg)
    got = host(lib.conv2d_int8(dev(x), dev(w), cfg.stride, cfg.pad))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("name", ["C2", "C4a"])
def test_conv_every_tile_and_split(lib, name):
    cfg = CONFIGS[name]
    x, w, want = oracle_conv(cfg)
    ksteps = layouts.packed_depth(cfg.C, cfg.R, cfg.S, 64) // 64
    for tile in range(lib.num_tiles()):
        steps = lib.tile_info(tile)[3]
        for split in (1, 3, 4):
            per = -(-ksteps // split)
            if ksteps % steps or per % steps:
                continue  # rejected combination, covered by test_gemm_every_tile_and_split
            assert lib.tile_applies(cfg.dims(), lib.LAYOUT_PACKED, 64, tile, split)
            got = run_layout(lib, cfg, x, w, "packed", 64, tile=tile, split_k=split)
            assert np.array_equal(got, want), f"tile {tile} split {split}"


BLOCK64 = [
    ConvShape("k-tail", 3, 128, 9, 9, 70, 3, 3, 1, 1), ConvShape("5x5-stride2", 1, 128, 13, 11, 64, 5, 5, 2, 2),
    ConvShape("1x5", 2, 128, 6, 20, 33, 1, 5, 1, 0), ConvShape("3x3-odd-blocks", 2, 192, 7, 7, 64, 3, 3, 1, 1),
    ConvShape("two-images-per-tile", 9, 64, 5, 5, 40, 2, 3, 1, 1), ConvShape("too-wide", 1, 128, 4, 140, 64, 3, 3, 1, 1),
    # five channel tiles x ten pixel tiles of 32 x 32 (both ragged): the blocked tile order with a narrower last group
    ConvShape("blocked-tile-order", 2, 64, 12, 13, 150, 3, 3, 1, 1),
]


@pytest.mark.parametrize("cfg", BLOCK64, ids=lambda c: c.name)
def test_conv_every_applicable_tile_64_channel_blocks(lib, cfg):
    """Every tile that accepts the problem, on small 64-channel-block shapes: ragged output channels
    and pixels, strides, tiles crossing image boundaries, odd and even step counts, one wide row."""
    x = uniform_int8(311, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(312, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    ran = 0
    for tile in range(lib.num_tiles()):
        if not lib.tile_applies(cfg.dims(), lib.LAYOUT_PACKED, 64, tile, 1):
            continue
        ran += 1
        got = run_layout(lib, cfg, x, w, "packed", 64, tile=tile, split_k=1)
        assert np.array_equal(got, want), f"tile {tile}: {np.count_nonzero(got != want)} mismatches"
    assert ran >= 10


# ---- the band kernel (window resident in LDS, depth split over the waves) ---------------------------
BAND_SHAPES = [
    CONFIGS["C4a"], CONFIGS["C2"],
    ConvShape("band-k-tail", 3, 128, 9, 9, 70, 3, 3, 1, 1),              # ragged output channels, 81-pixel images
    ConvShape("band-stride2", 1, 128, 13, 11, 64, 5, 5, 2, 2),           # 5x5 taps, stride 2: 50 steps -> falls outside (13 per wave)
    ConvShape("band-1x5", 2, 128, 6, 20, 33, 1, 5, 1, 0),                # one kernel row, ten steps: 3,3,3,1 per wave
    ConvShape("band-odd-blocks", 2, 192, 7, 7, 64, 3, 3, 1, 1),          # 27 steps: 7,7,7,6; 49 pixels
    ConvShape("band-short-last", 2, 64, 23, 14, 40, 3, 3, 1, 1),         # 23 output rows in bands of 7/8: a short last band
    ConvShape("band-one-step", 1, 64, 5, 5, 32, 1, 1, 1, 0),             # a single depth step: three idle waves
    ConvShape("band-two-steps", 2, 128, 6, 6, 16, 1, 1, 1, 0),           # fewer steps than waves, K below a row block
    ConvShape("band-wide", 1, 64, 4, 100, 64, 3, 3, 1, 1),               # one output row per band, 100 pixels of 128
    ConvShape("band-stride3", 1, 64, 20, 19, 48, 3, 2, 3, 1),            # stride 3 in both directions
    ConvShape("band-padded-channels", 1, 70, 10, 10, 32, 3, 3, 1, 1),    # 70 channels in two blocks of 64
    ConvShape("band-deep", 1, 512, 6, 6, 32, 3, 3, 1, 1),                # 72 steps: beyond twelve per wave
    ConvShape("band-too-wide", 1, 128, 4, 140, 64, 3, 3, 1, 1),          # an output row wider than the largest pixel tile
]


@pytest.mark.parametrize("cfg", BAND_SHAPES, ids=lambda c: c.name)
def test_band_kernel_shapes(lib, cfg):
    x, w = cfg.make() if cfg.name in CONFIGS else (uniform_int8(511, (cfg.N, cfg.C, cfg.H, cfg.W)), uniform_int8(512, (cfg.K, cfg.C, cfg.R, cfg.S)))
    applies = lib.tile_applies(cfg.dims(), lib.LAYOUT_PACKED, 64, lib.TILE_BAND, 1)
    assert applies == (cfg.name not in ("band-stride2", "band-deep", "band-too-wide"))
    if not applies:
        out = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
        with pytest.raises(lib.ConvError) as e:
            lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_PACKED, 64, lib.pack_layout(dev(x), 64, cfg.pad),
                                   lib.pack_weights(dev(w), lib.LAYOUT_PACKED, 64), out, tile=lib.TILE_BAND)
        assert e.value.status == lib.ERR_UNSUPPORTED
        return
    assert 0 < lib.tile_lds_bytes(cfg.dims(), lib.LAYOUT_PACKED, 64, lib.TILE_BAND, 1) <= 160 * 1024
    assert not lib.tile_applies(cfg.dims(), lib.LAYOUT_PACKED, 64, lib.TILE_BAND, 2)      # it has no depth split
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    got = run_layout(lib, cfg, x, w, "packed", 64, tile=lib.TILE_BAND)
    assert np.array_equal(got, want), f"{cfg.name}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("cfg", [c for c in BAND_SHAPES if c.name not in ("band-stride2", "band-deep", "band-too-wide")],
                         ids=lambda c: c.name)
def test_band_kernel_nhwc_result_and_activation(lib, cfg):
    """The band kernel's other two epilogues: the NHWC result (forced through the tile argument) and the activation + next layer's blocking (the GEMM stage picks
    its kernel itself there: for the benchmark shapes that is the band kernel).  Output channels that are not a
    multiple of four take the value-by-value stores."""
    x, w = cfg.make() if cfg.name in CONFIGS else (uniform_int8(511, (cfg.N, cfg.C, cfg.H, cfg.W)), uniform_int8(512, (cfg.K, cfg.C, cfg.R, cfg.S)))
    ref = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    xp = lib.pack_layout(dev(x), 64, cfg.pad); wp = lib.pack_weights(dev(w), lib.LAYOUT_PACKED, 64)
    want = layouts.unpack_nhwc(ref)
    buf = torch.full((want.size + 8,), -7, dtype=torch.int32, device=DEV)
    view = buf[4:4 + want.size].view(want.shape)     # (the entry point asks for a result on 16 bytes)
    lib.conv2d_int8_packed_nhwc(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, view, tile=lib.TILE_BAND)
    assert np.array_equal(host(view), want), cfg.name
    assert int(buf[3]) == -7 and int(buf[4 + want.size]) == -7
    for out_cb, out_pad, shift, relu in ((64, 1, 9, True), (16, 0, 7, False)):
        got = host(lib.conv2d_int8_packed_requant(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, out_cb, out_pad, shift, relu))
        np.testing.assert_array_equal(got, layouts.pack_layout(layouts.requant(ref, shift, relu), out_cb, out_pad), err_msg=cfg.name)


def test_band_kernel_other_layouts_and_dilation(lib):
    """It takes 64-channel blocks only (PAD_ONLY over exactly 64 channels is such a layout); kernel taps a
    dilation apart are address offsets into its window like any other."""
    cfg = ConvShape("band-pad-only", 2, 60, 9, 12, 40, 3, 3, 1, 1)
    x = uniform_int8(521, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(522, (cfg.K, cfg.C, cfg.R, cfg.S))
    assert lib.tile_applies(cfg.dims(), lib.LAYOUT_PAD_ONLY, 0, lib.TILE_BAND, 1)
    assert np.array_equal(run_layout(lib, cfg, x, w, "pad_only", 0, tile=lib.TILE_BAND), direct.conv2d_int8(x, w, 1, 1))
    for lname, cb in (("packed", 16), ("packed", 32), ("im2col", 0)):
        lay = {"packed": lib.LAYOUT_PACKED, "im2col": lib.LAYOUT_IM2COL}[lname]
        assert not lib.tile_applies(cfg.dims(), lay, cb, lib.TILE_BAND, 1)
    # the dilated layer of the benchmark's supplementary section at N = 4: the address-multiplier route picks
    # its GEMM-stage kernel itself; whichever it is, the result is the definition's
    dims, d = (4, 64, 28, 28, 64, 3, 3, 1, 2), 2
    x = uniform_int8(523, dims[:4]); w = uniform_int8(524, (64, 64, 3, 3))
    got = lib.conv2d_int8_dilated_direct(dims, d, dev(x), dev(w), 64)
    assert np.array_equal(host(got), direct.conv2d_int8_dilated(x, w, 1, 2, d))


def test_band_kernel_random_shapes(lib):
    rng = np.random.default_rng(9101)
    ran = 0
    while ran < 40:
        N = int(rng.integers(1, 4)); C = 64 * int(rng.integers(1, 5)); K = int(rng.choice([8, 32, 40, 64, 100]))
        R = int(rng.integers(1, 4)); S = int(rng.integers(1, 4)); st = int(rng.integers(1, 3)); pad = int(rng.integers(0, 3))
        H = int(rng.integers(3, 30)); W = int(rng.integers(3, 60))
        if R > H + 2 * pad or S > W + 2 * pad:
            continue
        cfg = ConvShape(f"b{ran}", N, C, H, W, K, R, S, st, pad)
        if not lib.tile_applies(cfg.dims(), lib.LAYOUT_PACKED, 64, lib.TILE_BAND, 1):
            continue
        ran += 1
        x = uniform_int8(600 + ran, (N, C, H, W)); w = uniform_int8(700 + ran, (K, C, R, S))
        got = run_layout(lib, cfg, x, w, "packed", 64, tile=lib.TILE_BAND)
        want = direct.conv2d_int8(x, w, st, pad)
        assert np.array_equal(got, want), f"{cfg.dims()}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("cfg", PAPER_SHAPES, ids=lambda c: c.name)
def test_conv_paper_table_shapes(lib, cfg):
    x, w, want = oracle_conv(cfg)
    got = host(lib.conv2d_int8(dev(x), dev(w), cfg.stride, cfg.pad))
    assert np.array_equal(got, want)
    for lname, cb in (("packed", 16), ("im2col", 0)):
        assert np.array_equal(run_layout(lib, cfg, x, w, lname, cb), want), lname


EDGE = [
    ConvShape("one-pixel", 1, 1, 1, 1, 1, 1, 1, 1, 0), ConvShape("P1Q1", 1, 2, 3, 4, 2, 5, 6, 1, 1),
    ConvShape("stride3", 2, 5, 10, 11, 3, 3, 2, 3, 1), ConvShape("wide-pad", 1, 3, 4, 4, 2, 3, 3, 1, 3),
    ConvShape("K1", 1, 17, 6, 6, 1, 3, 3, 1, 1), ConvShape("K33", 3, 33, 5, 7, 33, 2, 2, 2, 0),
    ConvShape("ragged", 1, 65, 13, 9, 70, 3, 3, 1, 1), ConvShape("tall-kernel", 1, 1, 30, 6, 4, 20, 5, 2, 0),
]


@pytest.mark.parametrize("cfg", EDGE, ids=lambda c: c.name)
def test_conv_edge_shapes(lib, cfg):
    x = uniform_int8(77, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(78, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    assert np.array_equal(host(lib.conv2d_int8(dev(x), dev(w), cfg.stride, cfg.pad)), want)
    for lname, cb in LAYOUT_CASES:
        assert np.array_equal(run_layout(lib, cfg, x, w, lname, cb), want), lname


def test_extreme_values(lib):
    """-128 * -128 in every tap: catches unsigned operands or a narrow product."""
    cfg = ConvShape("ext", 1, 64, 8, 8, 32, 3, 3, 1, 1)
    x = np.full((1, 64, 8, 8), -128, np.int8); w = np.full((32, 64, 3, 3), -128, np.int8)
    want = direct.conv2d_int8(x, w, 1, 1)
    assert want.max() == 64 * 9 * 16384
    assert np.array_equal(host(lib.conv2d_int8(dev(x), dev(w), 1, 1)), want)
    assert np.array_equal(run_layout(lib, cfg, x, w, "im2col", 0), want)


def test_ex_with_caller_workspace_and_prepacked_weights(lib):
    cfg = CONFIGS["C2"]
    x, w, want = oracle_conv(cfg)
    dx, dw = dev(x), dev(w)
    for lay, cb in ((lib.LAYOUT_PACKED, 64), (lib.LAYOUT_IM2COL, 0), (lib.LAYOUT_AUTO, 0)):
        ws = torch.empty(lib.conv2d_int8_workspace_bytes(cfg.dims(), lay, cb), dtype=torch.int8, device=DEV)
        out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
        lib.conv2d_int8_ex(cfg.dims(), lay, cb, dx, dw, out, ws)
        assert np.array_equal(host(out), want)
    wp = lib.pack_weights(dw, lib.LAYOUT_PACKED, 64)
    ws = torch.empty(lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_PACKED, 64, True),
                     dtype=torch.int8, device=DEV)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_PACKED, 64, dx, wp, out, ws, wt_is_packed=True)
    assert np.array_equal(host(out), want)
    small = torch.empty(256, dtype=torch.int8, device=DEV)
    with pytest.raises(lib.ConvError) as e:
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_PACKED, 64, dx, dw, out, small)
    assert e.value.status == lib.ERR_WORKSPACE


@pytest.mark.parametrize("dims,cb", [((1, 64, 6, 6, 1, 3, 3, 1, 1), 64), ((2, 128, 5, 7, 33, 3, 3, 1, 1), 64),
                                     ((1, 192, 6, 5, 100, 5, 5, 2, 2), 64), ((1, 64, 9, 9, 257, 1, 1, 1, 0), 16),
                                     ((1, 96, 7, 8, 70, 2, 3, 1, 1), 32), ((1, 64, 8, 8, 16, 5, 5, 1, 2), 64),
                                     ((1, 64, 12, 12, 20, 7, 7, 1, 3), 64), ((1, 80, 6, 6, 40, 3, 3, 1, 1), 64)], ids=str)
def test_fused_rewrite_weight_range(lib, dims, cb):
    """The weight half of the fused rewrite launch (channel blocking of KCRS, Table 2), one thread per 16 destination
    bytes: fewer pieces than a workgroup has threads, (k, channel block) pairs of 36 and 100 pieces that straddle
    workgroups, a ragged last workgroup, single-piece pairs (1x1, cb 16), large pairs (5x5 and 7x7, cb 64), and a
    channel count that is not whole blocks."""
    cfg = ConvShape("fused-w", *dims)
    assert lib.layout_applies(dims, lib.LAYOUT_PACKED, cb)
    x = uniform_int8(971, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(972, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    ws = torch.empty(lib.conv2d_int8_workspace_bytes(dims, lib.LAYOUT_PACKED, cb), dtype=torch.int8, device=DEV)
    out = torch.full(want.shape, -5, dtype=torch.int32, device=DEV)
    lib.conv2d_int8_ex(dims, lib.LAYOUT_PACKED, cb, dev(x), dev(w), out, ws)
    assert np.array_equal(host(out), want), f"{np.count_nonzero(host(out) != want)} mismatches"


def test_non_default_stream(lib):
    cfg = CONFIGS["C1"]
    x, w, want = oracle_conv(cfg)
    s = torch.cuda.Stream()
    dx, dw = dev(x), dev(w)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = lib.conv2d_int8(dx, dw, cfg.stride, cfg.pad)
    s.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)


# ---- the batch-scaled shapes bench.py times (supplementary section): sampled images -------------
def _sample_images(N, pixels=None, bytes_per_image=()):
    """About sixteen images of a batch: both ends and the middle; with `pixels` (output pixels per image) the
    images on both sides of several 256-pixel tile boundaries (the widest GEMM tile), near the start, the
    middle and the end of the pixel range; with per-image byte counts the last image below and the first
    image at or above byte offsets 2^31 and 2^32 of each such tensor."""
    pick = {0, 1, N // 2 - 1, N // 2, N - 2, N - 1}
    if pixels:
        tiles = N * pixels // 256
        for t in (1, 2, tiles // 3, tiles // 2, 2 * tiles // 3, tiles - 1):
            n = 256 * t // pixels            # the image that holds the tile's first pixel ...
            pick |= {n - 1, n, n + 1} if 256 * t % pixels else {n - 1, n}   # ... and its neighbours across the boundary
    for b in bytes_per_image:
        for limit in (1 << 31, 1 << 32):
            n = -(-limit // b)
            pick |= {n - 1, n}
    return sorted(n for n in pick if 0 <= n < N)


def test_batch_scaled_gemm_stage_sampled_images(lib):
    """C4a at N=2048 in the configuration bench.py times: whole output planes of sampled images
    against the direct convolution of those images (images are independent)."""
    cfg = CONFIGS["C4a"].scaled(2048)
    g = torch.Generator(device=DEV); g.manual_seed(4242)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
    lay, cb, _ = lib.select_layout(cfg.dims())
    xp = lib.pack_layout(x, cb, cfg.pad)
    wp = lib.pack_weights(w, lay, cb)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(cfg.dims(), lay, cb, xp, wp, out)
    wh = host(w)
    # (+ the last images of the batch: the partly filled last round of workgroups)
    picked = sorted(set(_sample_images(cfg.N, cfg.P * cfg.Q)) | set(range(cfg.N - 44, cfg.N - 39)) | {cfg.N - 2, cfg.N - 1})
    assert len(picked) >= 14
    for n in picked:
        want = direct.conv2d_int8(host(x[n:n + 1]), wh, cfg.stride, cfg.pad)
        assert np.array_equal(host(out[n:n + 1]), want), n
        assert np.array_equal(host(xp[n:n + 1]), layouts.pack_layout(host(x[n:n + 1]), cb, cfg.pad)), n


def test_offsets_past_32_bits(lib):
    """Batches whose tensors pass 2^31 and 2^32 bytes: the 64-channel 3x3 layer at N=10880 (NCHW input and
    blocked input past 2^31, int32 result past 2^33) through channel blocking + GEMM stage, and the
    three-channel stem at N=1400 (result past 2^32) through the stencil-unrolling GEMM stage.  Whole planes
    of the images on both sides of each limit, and of tile-straddling images, against the definition."""
    g = torch.Generator(device=DEV); g.manual_seed(4250)
    cfg = CONFIGS["C2"].scaled(10880)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
    xp = lib.pack_layout(x, 64, cfg.pad)
    wp = lib.pack_weights(w, lib.LAYOUT_PACKED, 64)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, out)
    wh = host(w)
    sizes = (cfg.C * cfg.H * cfg.W, xp[0].numel(), cfg.K * cfg.P * cfg.Q * 4)
    assert cfg.N * sizes[0] > 1 << 31 and cfg.N * sizes[1] > 1 << 31 and cfg.N * sizes[2] > 1 << 33
    for n in _sample_images(cfg.N, cfg.P * cfg.Q, sizes):
        xh = host(x[n:n + 1])
        assert np.array_equal(host(xp[n:n + 1]), layouts.pack_layout(xh, 64, cfg.pad)), ("pack", n)
        assert np.array_equal(host(out[n:n + 1]), direct.conv2d_int8(xh, wh, cfg.stride, cfg.pad)), ("gemm", n)
    del x, xp, out

    cfg = CONFIGS["C3"].scaled(1400)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, x, w, out, None)
    wh = host(w)
    assert out.numel() * 4 > 1 << 32
    for n in _sample_images(cfg.N, None, (cfg.K * cfg.P * cfg.Q * 4,)):
        assert np.array_equal(host(out[n:n + 1]), direct.conv2d_int8(host(x[n:n + 1]), wh, cfg.stride, cfg.pad)), ("stem", n)


def test_batch_scaled_layout_kernels_sampled_images(lib):
    g = torch.Generator(device=DEV); g.manual_seed(4243)
    cfg = CONFIGS["C2"].scaled(2048)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    xp = lib.pack_layout(x, 64, cfg.pad)
    for n in _sample_images(cfg.N):
        assert np.array_equal(host(xp[n:n + 1]), layouts.pack_layout(host(x[n:n + 1]), 64, cfg.pad)), n
    del x, xp
    cfg = CONFIGS["C3"].scaled(512)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    a = lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad)
    per = cfg.P * cfg.Q
    for n in _sample_images(cfg.N):
        want = layouts.im2col(host(x[n:n + 1]), cfg.R, cfg.S, cfg.stride, cfg.pad)
        assert np.array_equal(host(a[n * per:(n + 1) * per]), want), n


def test_batch_scaled_implicit_sampled_images(lib):
    """The stencil-unrolling GEMM stage at the batch sizes the benchmark times (C3 at N=512, C4b at
    N=2048): whole output planes of sampled images against the direct convolution of those images."""
    g = torch.Generator(device=DEV); g.manual_seed(4244)
    for name, scale in (("C3", 512), ("C4b", 2048)):
        cfg = CONFIGS[name].scaled(scale)
        x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
        w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
        out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, x, w, out, None)
        wh = host(w)
        for n in _sample_images(cfg.N):
            want = direct.conv2d_int8(host(x[n:n + 1]), wh, cfg.stride, cfg.pad)
            assert np.array_equal(host(out[n:n + 1]), want), (name, n)
        del x, out


def test_batch_scaled_newer_entries_sampled_images(lib):
    """The other batch-scaled lines of the benchmark, at its sizes: C4b at N=8192 (the 1x1 kernel's batch form),
    the three epilogues of the GEMM stage on C4a at N=2048, Image Pack of the C3 stem at N=4096, and the dilated
    3x3 layer at N=4096 by its three routes; whole planes of sampled images against the definitions."""
    g = torch.Generator(device=DEV); g.manual_seed(4245)
    cfg = CONFIGS["C4b"].scaled(8192)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, x, w, out, None)
    for n in _sample_images(cfg.N):
        assert np.array_equal(host(out[n:n + 1]), direct.conv2d_int8(host(x[n:n + 1]), host(w), 1, 0)), ("C4b", n)
    del x, out

    cfg = CONFIGS["C4a"].scaled(2048)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV, generator=g)
    xp = lib.pack_layout(x, 64, cfg.pad); wp = lib.pack_weights(w, lib.LAYOUT_PACKED, 64)
    onh = torch.empty((cfg.N, cfg.P, cfg.Q, cfg.K), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed_nhwc(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, onh)
    xact = lib.conv2d_int8_packed_requant(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, 64, 0, 9, True)
    for n in _sample_images(cfg.N):
        conv = direct.conv2d_int8(host(x[n:n + 1]), host(w), cfg.stride, cfg.pad)
        assert np.array_equal(host(onh[n:n + 1]), layouts.unpack_nhwc(conv)), ("nhwc", n)
        assert np.array_equal(host(xact[n:n + 1]), layouts.pack_layout(layouts.requant(conv, 9, True), 64, 0)), ("act", n)
    del x, xp, onh, xact

    cfg = CONFIGS["C3"].scaled(4096)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV, generator=g)
    x2 = lib.image_pack_int8(cfg.dims(), x)
    for n in _sample_images(cfg.N):
        assert np.array_equal(host(x2[n:n + 1]), layouts.image_pack(host(x[n:n + 1]), cfg.R, cfg.S, cfg.stride, cfg.pad)), ("ip", n)
    del x, x2

    dims, d = (4096, 64, 28, 28, 64, 3, 3, 1, 2), 2
    x = torch.randint(-128, 128, dims[:4], dtype=torch.int8, device=DEV, generator=g)
    w = torch.randint(-128, 128, (64, 64, 3, 3), dtype=torch.int8, device=DEV, generator=g)
    packed = lib.conv2d_int8_dilated(dims, d, x, w)
    direct_route = lib.conv2d_int8_dilated_direct(dims, d, x, w, 64)
    x2 = lib.dilation_pack_int8(dims, d, x)
    for n in _sample_images(dims[0]):
        want = direct.conv2d_int8_dilated(host(x[n:n + 1]), host(w), 1, 2, d)
        assert np.array_equal(host(packed[n:n + 1]), want), ("image pack route", n)
        assert np.array_equal(host(direct_route[n:n + 1]), want), ("address multiplier", n)
        assert np.array_equal(host(x2[4 * n:4 * n + 4]), layouts.dilation_pack(host(x[n:n + 1]), 2, d)), ("dilation pack", n)


# ---- the one-shot path called repeatedly and under graph replay ------------------------------------
def test_one_shot_back_to_back_and_mixed_shapes(lib):
    """Consecutive one-shot calls share the library's cached workspace: alternate shapes and layouts,
    twice over, and check every result afterwards."""
    names = ["C4a", "C2", "C1", "C4b", "C3", "C4a", "C4b", "C2"]
    data = {n: oracle_conv(CONFIGS[n]) for n in set(names)}
    dev_in = {n: (dev(data[n][0]), dev(data[n][1])) for n in data}
    outs = []
    for _ in range(2):
        for n in names:
            cfg = CONFIGS[n]
            outs.append((n, lib.conv2d_int8(dev_in[n][0], dev_in[n][1], cfg.stride, cfg.pad)))
    for n, o in outs:
        assert np.array_equal(host(o), data[n][2]), n


def test_one_shot_graph_replay(lib):
    """The benchmark replays captured one-shot calls: every replay must give the eager result, also with
    other work of the process in between."""
    cfgs = [CONFIGS["C4a"], CONFIGS["C4b"], CONFIGS["C2"]]
    data = [oracle_conv(c) for c in cfgs]
    ins = [(dev(x), dev(w)) for x, w, _ in data]
    outs = [torch.empty((c.N, c.K, c.P, c.Q), dtype=torch.int32, device=DEV) for c in cfgs]
    for c, (x, w), o in zip(cfgs, ins, outs):
        lib.conv2d_int8(x, w, c.stride, c.pad, out=o)       # eager first: sizes the cached workspace
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(3):
            for c, (x, w), o in zip(cfgs, ins, outs):
                lib.conv2d_int8(x, w, c.stride, c.pad, out=o)
    for rep in range(4):
        for o in outs:
            o.fill_(-1)
        g.replay()
        torch.cuda.synchronize()
        for (x, w, want), o in zip(data, outs):
            assert np.array_equal(o.cpu().numpy(), want), rep
        # eager work between replays, through the same path
        e = lib.conv2d_int8(ins[0][0], ins[0][1], cfgs[0].stride, cfgs[0].pad)
        assert np.array_equal(host(e), data[0][2])


def test_one_shot_workspace_growth_keeps_captured_graphs_valid(lib):
    """A graph captured while the cached workspace was small must still be valid after a larger problem has
    made the library move to a bigger block (the superseded block stays allocated); and a call that would
    have to grow the block while its stream is being captured is refused with nothing enqueued."""
    small, big = CONFIGS["C2"], ConvShape("grow", 192, 64, 56, 56, 64, 3, 3, 1, 1)       # 41 MB of rewritten input
    huge = ConvShape("grow2", 448, 64, 56, 56, 64, 3, 3, 1, 1)                           # 96 MB: beyond 2 x 41 MB
    x, w, want = oracle_conv(small)
    dx, dw = dev(x), dev(w)
    out = torch.empty((small.N, small.K, small.P, small.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8(dx, dw, small.stride, small.pad, out=out)         # eager first: sizes the cached workspace
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lib.conv2d_int8(dx, dw, small.stride, small.pad, out=out)
    gen = torch.Generator(device=DEV); gen.manual_seed(4260)
    bx = torch.randint(-128, 128, (huge.N, big.C, big.H, big.W), dtype=torch.int8, device=DEV, generator=gen)
    bw = torch.randint(-128, 128, (big.K, big.C, big.R, big.S), dtype=torch.int8, device=DEV, generator=gen)
    bout = lib.conv2d_int8(bx[:big.N], bw, big.stride, big.pad)       # grows the cache
    for n in (0, big.N - 1):
        assert np.array_equal(host(bout[n:n + 1]), direct.conv2d_int8(host(bx[n:n + 1]), host(bw), 1, 1)), n
    for rep in range(2):
        out.fill_(-1)
        g.replay()                                                    # still reads and writes the first block
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want), rep
    # growth under capture: refused, the capture goes on and what it holds is intact
    hout = torch.empty((huge.N, huge.K, huge.P, huge.Q), dtype=torch.int32, device=DEV)
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2):
        lib.conv2d_int8(dx, dw, small.stride, small.pad, out=out)
        with pytest.raises(lib.ConvError) as e:
            lib.conv2d_int8(bx, bw, huge.stride, huge.pad, out=hout)
        assert e.value.status == lib.ERR_WORKSPACE
    out.fill_(-1)
    g2.replay()
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    # outside capture the same call grows the block and runs
    lib.conv2d_int8(bx, bw, huge.stride, huge.pad, out=hout)
    n = huge.N - 1
    assert np.array_equal(host(hout[n:n + 1]), direct.conv2d_int8(host(bx[n:n + 1]), host(bw), 1, 1))


# ---- stencil unroll inside the GEMM stage ---------------------------------------------------
def run_implicit(lib, cfg, x, w, rewritten, dx=None):
    dx = dev(x) if dx is None else dx
    out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), 4321, dtype=torch.int32, device=DEV)
    if rewritten:
        lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dx, lib.pack_weights(dev(w), lib.LAYOUT_IMPLICIT, 0), out)
    else:
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dx, dev(w), out, None)
    return host(out)


@pytest.mark.parametrize("name", list(CONFIGS))
def test_implicit_configs(lib, name):
    cfg = CONFIGS[name]
    x, w, want = oracle_conv(cfg)
    if not lib.layout_applies(cfg.dims(), lib.LAYOUT_IMPLICIT):
        out = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
        with pytest.raises(lib.ConvError) as e:
            lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dev(x), dev(w), out, None)
        assert e.value.status == lib.ERR_UNSUPPORTED
        return
    for rewritten in (False, True):
        got = run_implicit(lib, cfg, x, w, rewritten)
        assert np.array_equal(got, want), f"{name} rewritten={rewritten}: {np.count_nonzero(got != want)} mismatches"


IMPLICIT_SHAPES = [
    ConvShape("row-tile-tail", 2, 3, 20, 150, 64, 7, 7, 2, 3), ConvShape("two-row-tile", 2, 3, 11, 90, 33, 3, 3, 2, 1),
    ConvShape("four-row-tile", 3, 4, 10, 30, 70, 3, 3, 1, 1), ConvShape("odd-width", 1, 2, 9, 13, 5, 3, 5, 1, 2),
    ConvShape("width-4", 1, 1, 6, 4, 3, 2, 2, 1, 1), ConvShape("1x1", 2, 5, 7, 9, 130, 1, 1, 1, 0),
    ConvShape("1x1-stride3", 1, 32, 10, 40, 8, 1, 1, 3, 0), ConvShape("tall", 1, 1, 40, 21, 32, 20, 5, 2, 0),
    ConvShape("wide-kernel", 1, 2, 6, 40, 9, 2, 9, 3, 4), ConvShape("deep-256", 1, 16, 8, 19, 40, 4, 4, 1, 2),
    ConvShape("one-pixel-out", 1, 3, 7, 7, 2, 7, 7, 1, 0), ConvShape("big-pad", 1, 1, 5, 6, 4, 3, 3, 2, 5),
    ConvShape("one-weight", 1, 1, 4, 4, 1, 1, 1, 1, 0),
    # 1x1 over whole 64-channel multiples (pixels turned around in LDS): ragged pixel and channel ends
    ConvShape("pw-64", 2, 64, 6, 6, 8, 1, 1, 1, 0), ConvShape("pw-192", 3, 192, 10, 14, 130, 1, 1, 1, 0),
    ConvShape("pw-512", 1, 512, 2, 2, 33, 1, 1, 1, 0), ConvShape("pw-320", 2, 320, 8, 16, 256, 1, 1, 1, 0),
    ConvShape("pw-448-wide", 1, 448, 1, 100, 5, 1, 1, 1, 0),
]


@pytest.mark.parametrize("cfg", IMPLICIT_SHAPES, ids=lambda c: c.name)
def test_implicit_shapes(lib, cfg):
    """All three tile shapes with ragged ends, strides, wide borders, image widths that are not a multiple
    of four, kernel rows of 1 to 9 taps, several output-channel blocks, both weight forms."""
    assert lib.layout_applies(cfg.dims(), lib.LAYOUT_IMPLICIT)
    x = uniform_int8(411, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(412, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    for rewritten in (False, True):
        got = run_implicit(lib, cfg, x, w, rewritten)
        assert np.array_equal(got, want), f"rewritten={rewritten}: {np.count_nonzero(got != want)} mismatches"


def test_implicit_unaligned_operands_and_forced_tiles(lib):
    cfg = ConvShape("unaligned", 2, 3, 12, 16, 5, 3, 3, 1, 1)
    x = uniform_int8(421, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(422, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    for off in (1, 2, 3):   # operands that start at any byte
        bx = torch.zeros(x.size + 8, dtype=torch.int8, device=DEV); bw = torch.zeros(w.size + 8, dtype=torch.int8, device=DEV)
        dx = bx[off:off + x.size].view(x.shape); dw = bw[off:off + w.size].view(w.shape)
        dx.copy_(dev(x)); dw.copy_(dev(w))
        out = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dx, dw, out, None)
        assert np.array_equal(host(out), want), off
    out = torch.zeros((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    wp = lib.pack_weights(dev(w), lib.LAYOUT_IMPLICIT, 0)
    for tile, split in ((0, 1), (-1, 2)):
        with pytest.raises(lib.ConvError) as e:
            lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dev(x), wp, out, tile=tile, split_k=split)
        assert e.value.status == lib.ERR_UNSUPPORTED


# ---- Image Pack (stride phases become channels) ----------------------------------------------
IMAGE_PACK_SHAPES = [
    ConvShape("ip-7x7-s2", 2, 3, 21, 23, 8, 7, 7, 2, 3), ConvShape("ip-20x5-s2", 1, 1, 41, 50, 32, 20, 5, 2, 0),
    ConvShape("ip-3x3-s3", 1, 16, 17, 19, 33, 3, 3, 3, 1), ConvShape("ip-1x1-s2", 2, 64, 9, 9, 8, 1, 1, 2, 0),
    ConvShape("ip-2x2-s2", 1, 4, 16, 16, 32, 2, 2, 2, 0), ConvShape("ip-5x4-s4", 1, 2, 30, 13, 5, 5, 4, 4, 2),
    ConvShape("ip-tiny", 1, 1, 3, 4, 2, 2, 2, 2, 1),          # fewer than 16 source bytes: the element-wise kernel
    ConvShape("ip-wide", 1, 1, 5, 16500, 2, 3, 3, 2, 1),      # a row too wide for the LDS tile: the element-wise kernel
    ConvShape("ip-tall", 1, 2, 400, 150, 4, 3, 3, 2, 1),      # planes cut into several row chunks
]


@pytest.mark.parametrize("cfg", IMAGE_PACK_SHAPES + [CONFIGS["C3"], CONFIGS["C5"]], ids=lambda c: c.name)
def test_image_pack(lib, cfg):
    """Both rewrites against their index maps, then the whole two-stage path in each inner layout."""
    x = uniform_int8(511, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(512, (cfg.K, cfg.C, cfg.R, cfg.S))
    np.testing.assert_array_equal(host(lib.image_pack_int8(cfg.dims(), dev(x))),
                                  layouts.image_pack(x, cfg.R, cfg.S, cfg.stride, cfg.pad))
    np.testing.assert_array_equal(host(lib.image_pack_weights(cfg.dims(), dev(w))), layouts.image_pack_weights(w, cfg.stride))
    want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    d2 = layouts.image_pack_dims(*cfg.dims())
    ran = 0
    for cb in (0, 16, 64):
        nbytes = lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_IMAGE_PACK, cb)
        out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), -3, dtype=torch.int32, device=DEV)
        if cb == 0 and not lib.layout_applies(d2, lib.LAYOUT_IMPLICIT):
            assert nbytes == 0
            with pytest.raises(lib.ConvError) as e:
                lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMAGE_PACK, cb, dev(x), dev(w), out,
                                   torch.empty(1 << 20, dtype=torch.int8, device=DEV))
            assert e.value.status == lib.ERR_UNSUPPORTED
            continue
        ws = torch.empty(nbytes + 256, dtype=torch.int8, device=DEV)
        ws = ws[(-ws.data_ptr()) % 256:]
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMAGE_PACK, cb, dev(x), dev(w), out, ws)
        assert np.array_equal(host(out), want), f"inner cb {cb}: {np.count_nonzero(host(out) != want)} mismatches"
        ran += 1
    assert ran >= 2
    # a workspace one byte short is refused before anything runs
    with pytest.raises(lib.ConvError) as e:
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMAGE_PACK, 16, dev(x), dev(w), out,
                           ws[:lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_IMAGE_PACK, 16) - 1])
    assert e.value.status == lib.ERR_WORKSPACE


# ---- seeded random shapes through the kernels that stage their own operands -----------------------
def _random_shapes(seed, count, want):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        N = int(rng.integers(1, 4)); C = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 64, 128])); K = int(rng.choice([1, 7, 32, 40, 65, 130]))
        R = int(rng.integers(1, 8)); S = int(rng.integers(1, 10)); st = int(rng.integers(1, 5)); pad = int(rng.integers(0, 5))
        H = int(rng.integers(1, 24)); W = int(rng.integers(1, 150))
        if R > H + 2 * pad or S > W + 2 * pad:
            continue
        dims = (N, C, H, W, K, R, S, st, pad)
        if want(dims):
            out.append(ConvShape(f"r{len(out)}", *dims))
    return out


def test_implicit_random_shapes(lib):
    shapes = _random_shapes(9001, 60, lambda d: lib.layout_applies(d, lib.LAYOUT_IMPLICIT) and d[0] * d[4] * d[2] * d[3] < 400000)
    rng = np.random.default_rng(9003)   # the 1x1 form has a narrow domain: drawn from inside it
    while len(shapes) < 75:
        dims = (int(rng.integers(1, 4)), 64 * int(rng.integers(1, 9)), int(rng.integers(1, 12)), int(rng.integers(1, 40)),
                int(rng.choice([1, 31, 32, 100, 129, 260])), 1, 1, 1, 0)
        if lib.layout_applies(dims, lib.LAYOUT_IMPLICIT):
            shapes.append(ConvShape(f"p{len(shapes)}", *dims))
    for cfg in shapes:
        x = uniform_int8(cfg.H * 131 + cfg.W, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(cfg.K * 17 + cfg.C, (cfg.K, cfg.C, cfg.R, cfg.S))
        want = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
        for rewritten in (False, True):
            got = run_implicit(lib, cfg, x, w, rewritten)
            assert np.array_equal(got, want), f"{cfg.dims()} rewritten={rewritten}: {np.count_nonzero(got != want)} mismatches"


def test_image_pack_random_shapes(lib):
    shapes = _random_shapes(9002, 30, lambda d: d[7] > 1 and d[1] <= 16 and d[0] * d[4] * d[2] * d[3] < 400000)
    for cfg in shapes:
        x = uniform_int8(cfg.H * 31 + cfg.W, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(cfg.K * 7 + cfg.C, (cfg.K, cfg.C, cfg.R, cfg.S))
        np.testing.assert_array_equal(host(lib.image_pack_int8(cfg.dims(), dev(x))),
                                      layouts.image_pack(x, cfg.R, cfg.S, cfg.stride, cfg.pad), err_msg=str(cfg.dims()))
        np.testing.assert_array_equal(host(lib.image_pack_weights(cfg.dims(), dev(w))),
                                      layouts.image_pack_weights(w, cfg.stride), err_msg=str(cfg.dims()))
        nbytes = lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_IMAGE_PACK, 16)
        ws = torch.empty(nbytes + 256, dtype=torch.int8, device=DEV); ws = ws[(-ws.data_ptr()) % 256:]
        out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), -3, dtype=torch.int32, device=DEV)
        lib.conv2d_int8_ex(cfg.dims(), lib.LAYOUT_IMAGE_PACK, 16, dev(x), dev(w), out, ws)
        assert np.array_equal(host(out), direct.conv2d_int8(x, w, cfg.stride, cfg.pad)), cfg.dims()


# ---- NHWC tensors -------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(2, 5, 3, 4), (1, 64, 14, 14), (3, 33, 7, 9), (1, 1, 1, 1), (2, 130, 1, 37)])
def test_unpack_nhwc(lib, shape):
    o = (np.arange(int(np.prod(shape)), dtype=np.int64) * 2654435761 % (1 << 31) - (1 << 30)).astype(np.int32).reshape(shape)
    np.testing.assert_array_equal(host(lib.unpack_nhwc_int32(dev(o))), layouts.unpack_nhwc(o))


@pytest.mark.parametrize("cfg", [CONFIGS["C1"], CONFIGS["C2"], CONFIGS["C4a"], CONFIGS["C4b"], CONFIGS["C3"],
                                 ConvShape("nhwc-ragged", 2, 37, 9, 11, 21, 3, 2, 2, 1),
                                 ConvShape("nhwc-deep", 1, 256, 7, 7, 64, 3, 3, 1, 1),      # small and deep: a depth split
                                 ConvShape("nhwc-k130", 1, 32, 12, 12, 130, 3, 3, 1, 1),
                                 ConvShape("nhwc-1x1-k70", 3, 128, 7, 9, 70, 1, 1, 1, 0),   # 1x1: a plain matrix product, one launch
                                 ConvShape("nhwc-1x1-s2", 2, 64, 9, 9, 32, 1, 1, 2, 0),     # 1x1 with a stride: not that form
                                 # 1x1 on a grid too small for the chip: the depth split over a workgroup's waves (every C / 128,
                                 # pixels ragged against 32 and against 8, channels against 32, one pixel, four channels)
                                 ConvShape("nhwc-1x1-split-128", 3, 128, 7, 9, 72, 1, 1, 1, 0),
                                 ConvShape("nhwc-1x1-split-256", 2, 256, 3, 5, 4, 1, 1, 1, 0),
                                 ConvShape("nhwc-1x1-split-384", 1, 384, 1, 1, 36, 1, 1, 1, 0),
                                 ConvShape("nhwc-1x1-split-512", 1, 512, 5, 5, 100, 1, 1, 1, 0),
                                 ConvShape("nhwc-1x1-split-most", 2, 128, 14, 14, 1248, 1, 1, 1, 0)],   # 13 x 39 workgroups: just inside its bound
                         ids=lambda c: c.name)
def test_conv_nhwc_one_shot(lib, cfg):
    """NHWC in, NHWC out: the NCHW definition seen through transposed views.  The GEMM stage writes NHWC
    itself; a result that does not start on 16 bytes takes the staging tensor and the unpacking pass."""
    x = uniform_int8(611, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(612, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = layouts.unpack_nhwc(direct.conv2d_int8(x, w, cfg.stride, cfg.pad))
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    got = host(lib.conv2d_int8_nhwc(dev(xh), dev(w), cfg.stride, cfg.pad))
    assert got.shape == want.shape and np.array_equal(got, want)
    buf = torch.full((want.size + 4,), -3, dtype=torch.int32, device=DEV)
    view = buf[1:1 + want.size].view(want.shape)
    lib.conv2d_int8_nhwc(dev(xh), dev(w), cfg.stride, cfg.pad, out=view)
    assert np.array_equal(host(view), want) and int(buf[0]) == -3 and int(buf[-1]) == -3


NHWC_WINDOW_SHAPES = [
    ConvShape("nhwc-stem", 2, 3, 40, 52, 64, 7, 7, 2, 3),          # the C3 kind: S*C = 21 bytes per kernel row
    ConvShape("nhwc-speech", 1, 1, 61, 90, 32, 20, 5, 2, 0),       # the C5 kind: one channel
    ConvShape("nhwc-k70", 1, 5, 17, 23, 70, 3, 3, 1, 1),           # two channel blocks, the second ragged; K % 4 != 0
    ConvShape("nhwc-k7", 3, 2, 9, 40, 7, 5, 4, 3, 2),              # fewer channels than one dword of results
    ConvShape("nhwc-wide", 1, 4, 6, 300, 16, 3, 5, 1, 2),          # several tiles per row and a ragged last one
    ConvShape("nhwc-c13", 1, 13, 12, 12, 32, 2, 3, 1, 0),          # S*C = 39: a kernel row that is not whole dwords
]


@pytest.mark.parametrize("cfg", NHWC_WINDOW_SHAPES, ids=lambda c: c.name)
def test_conv_nhwc_unrolling_kernel(lib, cfg):
    """Shapes the selector gives to the kernel that unrolls the stencil itself, from an NHWC source (Sec. 5.2):
    depth order (r, s, c), KCRS weights reordered inside the kernel, NHWC result.  One launch: the cached
    workspace is not touched."""
    assert lib.select_layout(cfg.dims())[0] == lib.LAYOUT_IMPLICIT and cfg.R * (-(-cfg.S * cfg.C // 4) * 4) <= 256
    x = uniform_int8(711, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(712, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = layouts.unpack_nhwc(direct.conv2d_int8(x, w, cfg.stride, cfg.pad))
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    got = host(lib.conv2d_int8_nhwc(dev(xh), dev(w), cfg.stride, cfg.pad))
    assert got.shape == want.shape and np.array_equal(got, want)
    buf = torch.full((want.size + 4,), -3, dtype=torch.int32, device=DEV)   # a result that starts on 4 bytes only
    view = buf[1:1 + want.size].view(want.shape)
    lib.conv2d_int8_nhwc(dev(xh), dev(w), cfg.stride, cfg.pad, out=view)
    assert np.array_equal(host(view), want) and int(buf[0]) == -3 and int(buf[-1]) == -3


def test_conv_nhwc_unrolling_kernel_random_shapes(lib):
    rng = np.random.default_rng(8128)
    done = 0
    for _ in range(400):
        if done == 24:
            break
        C = int(rng.choice([1, 2, 3, 4, 5, 7, 12])); R = int(rng.integers(1, 8)); S = int(rng.integers(1, 8))
        st = int(rng.integers(1, 4)); pad = int(rng.integers(0, 4)); K = int(rng.choice([3, 16, 32, 33, 64, 100]))
        H = int(rng.integers(R, 30)); W = int(rng.integers(max(S, 2), 80)); N = int(rng.integers(1, 3))
        cfg = ConvShape("r", N, C, H, W, K, R, S, st, pad)
        if cfg.P < 1 or cfg.Q < 1 or W * C < 4 or R * (-(-S * C // 4) * 4) > 256:
            continue
        if lib.select_layout(cfg.dims())[0] != lib.LAYOUT_IMPLICIT:
            continue
        x = uniform_int8(7000 + done, (N, C, H, W)); w = uniform_int8(7100 + done, (K, C, R, S))
        want = layouts.unpack_nhwc(direct.conv2d_int8(x, w, st, pad))
        got = host(lib.conv2d_int8_nhwc(dev(np.ascontiguousarray(x.transpose(0, 2, 3, 1))), dev(w), st, pad))
        assert np.array_equal(got, want), cfg.dims()
        done += 1
    assert done == 24


# ---- activation between layers -------------------------------------------------------------------
@pytest.mark.parametrize("shift,relu", [(0, False), (0, True), (1, False), (7, True), (10, False), (31, False)])
def test_requant(lib, shift, relu):
    rng = np.random.default_rng(700 + shift)
    x = rng.integers(-2 ** 31, 2 ** 31, size=(3, 5, 7, 11), dtype=np.int64).astype(np.int32)
    x.reshape(-1)[:8] = [0, -1, 2 ** 31 - 1, -2 ** 31, 1 << max(shift - 1, 0), -(1 << max(shift - 1, 0)), 127 << shift if shift < 24 else 5, -128]
    small = rng.integers(-(300 << min(shift, 20)), 300 << min(shift, 20), size=x.shape, dtype=np.int64).astype(np.int32)
    for t in (x, small):
        np.testing.assert_array_equal(host(lib.requant_int8(dev(t), shift, relu)), layouts.requant(t, shift, relu))
        for cb, pad in ((16, 1), (64, 0)):
            want = layouts.pack_layout(layouts.requant(t, shift, relu), cb, pad)
            np.testing.assert_array_equal(host(lib.requant_pack_layout(dev(t), cb, pad, shift, relu)), want)


def test_chained_layers_stay_blocked(lib):
    """C4a, activation, C4b with the intermediate never leaving the blocked layout: the second layer's GEMM
    stage consumes what requant_pack_layout wrote.  Checked against convolution, activation, convolution
    by definition."""
    a, b = CONFIGS["C4a"], CONFIGS["C4b"]
    assert (a.N, a.K, a.P, a.Q) == (b.N, b.C, b.H, b.W)
    x, w1, mid = oracle_conv(a)
    w2 = uniform_int8(801, (b.K, b.C, b.R, b.S))
    shift, relu = 9, True
    act = layouts.requant(mid, shift, relu)
    assert 0 < np.count_nonzero(act) and act.max() == 127 and len(np.unique(act)) > 100   # the activation is exercised
    want = direct.conv2d_int8(act, w2, b.stride, b.pad)
    out1 = lib.conv2d_int8(dev(x), dev(w1), a.stride, a.pad)
    xq = lib.requant_pack_layout(out1, 64, b.pad, shift, relu)
    wq = lib.pack_weights(dev(w2), lib.LAYOUT_PACKED, 64)
    out2 = torch.empty((b.N, b.K, b.P, b.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(b.dims(), lib.LAYOUT_PACKED, 64, xq, wq, out2)
    assert np.array_equal(host(out2), want)


# ---- dilated convolution: sub-images into the batch, dense convolution, interleaving (Sec. 6.1) ------------
DILATED_SHAPES = [
    # (N, C, H, W, K, R, S, stride, pad), dilation
    ((4, 64, 28, 28, 64, 3, 3, 1, 2), 2),     # "same"-size 3x3, dilation 2
    ((2, 16, 33, 65, 40, 3, 3, 1, 4), 4),     # sub-images one row short of each other (41 x 73 padded)
    ((1, 3, 37, 41, 8, 5, 3, 1, 0), 3),       # low channel count, no padding
    ((2, 1, 9, 50, 32, 2, 2, 1, 1), 2),
    ((1, 128, 14, 14, 130, 3, 3, 1, 2), 2),   # ragged output channels
    ((1, 2, 6, 5, 2, 1, 1, 1, 1), 2),         # 1x1: the dilation changes nothing but the route
    ((1, 4, 20, 20, 4, 3, 3, 1, 7), 7),       # a plane smaller than one block, odd extents
    ((1, 2, 301, 203, 3, 3, 3, 1, 1), 2),     # planes cut into several row chunks, odd plane size
    ((1, 1, 3, 5, 2, 2, 2, 1, 1), 2),         # fewer than 16 source bytes: the element-wise kernel
    ((1, 1, 4, 8300, 2, 1, 3, 1, 0), 2),      # a row too wide for the LDS tile: the element-wise kernel
]


@pytest.mark.parametrize("case", DILATED_SHAPES, ids=str)
def test_dilated_convolution(lib, case):
    dims, d = case
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(901, (N, C, H, W)); w = uniform_int8(902, (K, C, R, S))
    # the two rewrites against their index maps
    x2 = lib.dilation_pack_int8(dims, d, dev(x))
    np.testing.assert_array_equal(host(x2), layouts.dilation_pack(x, pad, d))
    d2 = layouts.dilation_dims(N, C, H, W, K, R, S, pad, d)
    P, Q = direct.out_hw_dilated(H, W, R, S, 1, pad, d)
    P2, Q2 = d2[2] - R + 1, d2[3] - S + 1
    o2 = (np.arange(d2[0] * K * P2 * Q2, dtype=np.int64) * 2654435761 % (1 << 31) - (1 << 30)).astype(np.int32).reshape(d2[0], K, P2, Q2)
    np.testing.assert_array_equal(host(lib.dilation_unpack_int32(dims, d, dev(o2))), layouts.dilation_unpack(o2, d, P, Q))
    # the whole path against the definition, in every layout the dense problem can run in
    want = direct.conv2d_int8_dilated(x, w, 1, pad, d)
    ran = 0
    for layout, cb in ((lib.LAYOUT_AUTO, 0), (lib.LAYOUT_PACKED, 16), (lib.LAYOUT_PACKED, 64), (lib.LAYOUT_IM2COL, 0),
                       (lib.LAYOUT_PAD_ONLY, 0), (lib.LAYOUT_IMPLICIT, 0)):
        if layout == lib.LAYOUT_IMPLICIT and not lib.layout_applies(d2, lib.LAYOUT_IMPLICIT):
            assert lib.conv2d_int8_dilated_workspace_bytes(dims, d, layout, cb) == 0
            continue
        out = torch.full((N, K, P, Q), -3, dtype=torch.int32, device=DEV)
        lib.conv2d_int8_dilated(dims, d, dev(x), dev(w), layout, cb, out=out)
        assert np.array_equal(host(out), want), f"{lib.LAYOUT_NAMES[layout]} cb {cb}: {np.count_nonzero(host(out) != want)} mismatches"
        ran += 1
    assert ran >= 5
    # the paper's reference for a dilated layer -- the kernel spread out with zeros, run densely -- agrees
    ws = np.zeros((K, C, d * (R - 1) + 1, d * (S - 1) + 1), dtype=np.int8)
    ws[:, :, ::d, ::d] = w
    assert np.array_equal(host(lib.conv2d_int8(dev(x), dev(ws), 1, pad)), want)


def test_dilation_pack_unaligned_destination(lib):
    """Planes of odd size, and a destination that does not start on a dword: byte stores."""
    dims, d = (2, 3, 9, 7, 4, 3, 3, 1, 1), 2
    x = uniform_int8(903, dims[:4])
    want = layouts.dilation_pack(x, 1, d)
    buf = torch.zeros(want.size + 16, dtype=torch.int8, device=DEV)
    for off in (0, 1, 2, 3):
        view = buf[off:off + want.size].view(want.shape)
        lib.dilation_pack_int8(dims, d, dev(x), out=view)
        np.testing.assert_array_equal(host(view), want)


# ---- activation fused into the GEMM stage's epilogue ------------------------------------------------------
FUSED_ACT_SHAPES = [
    ConvShape("fa-3x3", 2, 64, 14, 14, 128, 3, 3, 1, 1), ConvShape("fa-ragged", 1, 20, 9, 11, 37, 3, 2, 1, 1),
    ConvShape("fa-stride", 2, 16, 17, 15, 65, 3, 3, 2, 1), ConvShape("fa-1x1", 1, 128, 7, 7, 256, 1, 1, 1, 0),
    ConvShape("fa-k3", 1, 8, 6, 5, 3, 3, 3, 1, 1),
]


@pytest.mark.parametrize("cfg", FUSED_ACT_SHAPES + [CONFIGS["C1"], CONFIGS["C2"], CONFIGS["C4a"]], ids=lambda c: c.name)
def test_gemm_stage_with_fused_activation(lib, cfg):
    x = uniform_int8(931, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(932, (cfg.K, cfg.C, cfg.R, cfg.S))
    conv = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    for layout, cb in ((lib.LAYOUT_PACKED, 16), (lib.LAYOUT_PACKED, 64), (lib.LAYOUT_IM2COL, 0)):
        xp = lib.im2col_int8(dev(x), cfg.R, cfg.S, cfg.stride, cfg.pad) if layout == lib.LAYOUT_IM2COL else lib.pack_layout(dev(x), cb, cfg.pad)
        wp = lib.pack_weights(dev(w), layout, cb)
        for out_cb, out_pad, shift, relu in ((64, 0, 9, True), (16, 1, 7, False), (32, 2, 0, True)):
            want = layouts.pack_layout(layouts.requant(conv, shift, relu), out_cb, out_pad)
            out = torch.full(want.shape, 77, dtype=torch.int8, device=DEV)   # stale contents must not survive
            lib.conv2d_int8_packed_requant(cfg.dims(), layout, cb, xp, wp, out_cb, out_pad, shift, relu, out=out)
            got = host(out)
            assert np.array_equal(got, want), f"{lib.LAYOUT_NAMES[layout]} cb {cb} -> cb {out_cb} pad {out_pad} shift {shift}: " \
                                              f"{np.count_nonzero(got != want)} mismatches"


def test_chained_layers_with_fused_activation(lib):
    """C4a with the activation in its epilogue hands C4b its blocked input directly: two GEMM-stage launches."""
    a, b = CONFIGS["C4a"], CONFIGS["C4b"]
    x, w1, mid = oracle_conv(a)
    w2 = uniform_int8(801, (b.K, b.C, b.R, b.S))
    shift, relu = 9, True
    want = direct.conv2d_int8(layouts.requant(mid, shift, relu), w2, b.stride, b.pad)
    xq1 = lib.pack_layout(dev(x), 64, a.pad)
    wq1 = lib.pack_weights(dev(w1), lib.LAYOUT_PACKED, 64)
    xq2 = lib.conv2d_int8_packed_requant(a.dims(), lib.LAYOUT_PACKED, 64, xq1, wq1, 64, b.pad, shift, relu)
    wq2 = lib.pack_weights(dev(w2), lib.LAYOUT_PACKED, 64)
    out2 = torch.empty((b.N, b.K, b.P, b.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(b.dims(), lib.LAYOUT_PACKED, 64, xq2, wq2, out2)
    assert np.array_equal(host(out2), want)


def test_mfma_probe_is_linear_in_its_iteration_count(lib):
    """The probe adds the same operand product every iteration: checksums scale with the count (mod 2^32)."""
    one, ops1 = lib.mfma_probe_int8(4, 1)
    three, ops3 = lib.mfma_probe_int8(4, 3)
    a, b = host(one).astype(np.int64), host(three).astype(np.int64)
    assert ops3 == 3 * ops1 == 3 * 2 * 32768 * 16 * 4
    assert np.count_nonzero(a) > a.size // 2
    assert np.array_equal((3 * a) & 0xFFFFFFFF, b & 0xFFFFFFFF)


DIRECT_DILATED = DILATED_SHAPES[:8] + [((2, 16, 33, 40, 24, 3, 3, 2, 3), 3), ((1, 70, 21, 19, 9, 2, 3, 3, 2), 2),
                                       ((1, 8, 12, 12, 4, 3, 3, 1, 1), 1)]


@pytest.mark.parametrize("case", DIRECT_DILATED, ids=str)
def test_dilated_convolution_as_an_address_multiplier(lib, case):
    """Strides and dilations together, against the definition."""
    dims, d = case
    N, C, H, W, K, R, S, st, pad = dims
    x = uniform_int8(941, (N, C, H, W)); w = uniform_int8(942, (K, C, R, S))
    want = direct.conv2d_int8_dilated(x, w, st, pad, d)
    for cb in (0, 16, 64):
        out = torch.full(want.shape, -3, dtype=torch.int32, device=DEV)
        lib.conv2d_int8_dilated_direct(dims, d, dev(x), dev(w), cb, out=out)
        assert np.array_equal(host(out), want), f"cb {cb}: {np.count_nonzero(host(out) != want)} mismatches"


@pytest.mark.parametrize("dims", [(520, 64, 14, 14, 40, 1, 1, 1, 0), (300, 128, 14, 14, 200, 1, 1, 1, 0),
                                  (140, 64, 30, 30, 32, 1, 1, 1, 0), (64, 192, 56, 56, 33, 1, 1, 1, 0),
                                  (512, 64, 2, 106, 16, 1, 1, 1, 0)], ids=str)
def test_pointwise_batch_form(lib, dims):
    """Batches large enough for the 1x1 kernel that owns up to 224 pixels of an image per workgroup:
    whole 14x14 images, several pixel ranges per image with a short last one, ragged output channels."""
    cfg = ConvShape("pw-batch", *dims)
    assert lib.layout_applies(dims, lib.LAYOUT_IMPLICIT)
    x = uniform_int8(951, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(952, (cfg.K, cfg.C, 1, 1))
    want = direct.conv2d_int8(x, w, 1, 0)
    for rewritten in (False, True):
        got = run_implicit(lib, cfg, x, w, rewritten)
        assert np.array_equal(got, want), f"rewritten={rewritten}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("dims", [(8, 512, 14, 14, 128, 1, 1, 1, 0), (1, 512, 14, 14, 1024, 1, 1, 1, 0), (1, 128, 14, 14, 33, 1, 1, 1, 0),
                                  (2, 256, 5, 4, 70, 1, 1, 1, 0), (1, 384, 1, 36, 1, 1, 1, 1, 0),
                                  (3, 512, 2, 2, 257, 1, 1, 1, 0), (7, 128, 3, 12, 31, 1, 1, 1, 0),
                                  (1, 256, 9, 28, 64, 1, 1, 1, 0)], ids=str)
def test_pointwise_split_depth_form(lib, dims):
    """Few pixel tiles (below half the chip's compute units) and C % 128 = 0: the 1x1 kernel whose four waves share
    the depth and add their partial blocks up through LDS.  The headline 1x1 layer itself (eight images, 128 output
    channels) and its transpose in batch and channels, every C / 128, output
    channels ragged against 32 and against 8 (a single one too), pixel tiles ragged against 32, images of one tile
    and of four pixels."""
    cfg = ConvShape("pw-split", *dims)
    assert lib.layout_applies(dims, lib.LAYOUT_IMPLICIT)
    x = uniform_int8(961, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(962, (cfg.K, cfg.C, 1, 1))
    want = direct.conv2d_int8(x, w, 1, 0)
    for rewritten in (False, True):
        got = run_implicit(lib, cfg, x, w, rewritten)
        assert np.array_equal(got, want), f"rewritten={rewritten}: {np.count_nonzero(got != want)} mismatches"
    np.testing.assert_array_equal(host(lib.conv2d_int8(dev(x), dev(w), 1, 0)), want)


# ---- seeded random shapes through the routes added around the GEMM stage's epilogue ---------------------------
def test_dilated_random_shapes(lib):
    rng = np.random.default_rng(9101)
    done = 0
    while done < 40:
        N = int(rng.integers(1, 4)); C = int(rng.choice([1, 3, 8, 16, 40, 64])); K = int(rng.choice([1, 7, 32, 65]))
        R = int(rng.integers(1, 5)); S = int(rng.integers(1, 5)); d = int(rng.integers(2, 6)); pad = int(rng.integers(0, 6))
        st = int(rng.integers(1, 4)); H = int(rng.integers(1, 40)); W = int(rng.integers(1, 70))
        if d * (R - 1) + 1 > H + 2 * pad or d * (S - 1) + 1 > W + 2 * pad:
            continue
        x = uniform_int8(H * 37 + W, (N, C, H, W)); w = uniform_int8(K * 11 + C, (K, C, R, S))
        dims = (N, C, H, W, K, R, S, st, pad)
        want = direct.conv2d_int8_dilated(x, w, st, pad, d)
        got = host(lib.conv2d_int8_dilated_direct(dims, d, dev(x), dev(w)))
        assert np.array_equal(got, want), f"address multiplier {dims} d={d}"
        if st == 1:
            np.testing.assert_array_equal(host(lib.dilation_pack_int8(dims, d, dev(x))), layouts.dilation_pack(x, pad, d), err_msg=str((dims, d)))
            for layout, cb in ((lib.LAYOUT_AUTO, 0), (lib.LAYOUT_PACKED, 16), (lib.LAYOUT_IM2COL, 0)):
                got = host(lib.conv2d_int8_dilated(dims, d, dev(x), dev(w), layout, cb))
                assert np.array_equal(got, want), f"image pack route {dims} d={d} {lib.LAYOUT_NAMES[layout]}"
        done += 1


def test_fused_activation_and_nhwc_random_shapes(lib):
    shapes = _random_shapes(9102, 30, lambda d: d[0] * d[4] * d[2] * d[3] < 300000)
    rng = np.random.default_rng(9103)
    for cfg in shapes:
        x = uniform_int8(cfg.H * 13 + cfg.W, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(cfg.K * 5 + cfg.C, (cfg.K, cfg.C, cfg.R, cfg.S))
        conv = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
        xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
        assert np.array_equal(host(lib.conv2d_int8_nhwc(dev(xh), dev(w), cfg.stride, cfg.pad)), layouts.unpack_nhwc(conv)), cfg.dims()
        cb = int(rng.choice([16, 32, 64])); out_cb = int(rng.choice([16, 32, 64])); out_pad = int(rng.integers(0, 3))
        shift = int(rng.integers(0, 14)); relu = bool(rng.integers(0, 2))
        xp = lib.pack_layout(dev(x), cb, cfg.pad); wp = lib.pack_weights(dev(w), lib.LAYOUT_PACKED, cb)
        want = layouts.pack_layout(layouts.requant(conv, shift, relu), out_cb, out_pad)
        got = host(lib.conv2d_int8_packed_requant(cfg.dims(), lib.LAYOUT_PACKED, cb, xp, wp, out_cb, out_pad, shift, relu))
        assert np.array_equal(got, want), (cfg.dims(), cb, out_cb, out_pad, shift, relu)


@pytest.mark.parametrize("cfg", [CONFIGS["C1"], CONFIGS["C3"], CONFIGS["C5"], CONFIGS["C4b"],
                                 ConvShape("ia-ragged", 2, 3, 19, 37, 21, 5, 3, 2, 2), ConvShape("ia-1x1", 3, 128, 6, 10, 70, 1, 1, 1, 0),
                                 ConvShape("ia-batch", 300, 64, 14, 14, 40, 1, 1, 1, 0)], ids=lambda c: c.name)
def test_implicit_kernels_with_fused_activation(lib, cfg):
    """The two kernels that read NCHW themselves, with the activation in their epilogue."""
    assert lib.layout_applies(cfg.dims(), lib.LAYOUT_IMPLICIT)
    x = uniform_int8(961, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(962, (cfg.K, cfg.C, cfg.R, cfg.S))
    conv = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    wp = lib.pack_weights(dev(w), lib.LAYOUT_IMPLICIT, 0)
    for out_cb, out_pad, shift, relu in ((64, 0, 6, True), (16, 1, 4, False), (32, 2, 0, True)):
        want = layouts.pack_layout(layouts.requant(conv, shift, relu), out_cb, out_pad)
        out = torch.full(want.shape, 77, dtype=torch.int8, device=DEV)
        lib.conv2d_int8_packed_requant(cfg.dims(), lib.LAYOUT_IMPLICIT, 0, dev(x), wp, out_cb, out_pad, shift, relu, out=out)
        got = host(out)
        assert np.array_equal(got, want), f"-> cb {out_cb} pad {out_pad} shift {shift}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("cfg", [CONFIGS["C2"], CONFIGS["C4a"], ConvShape("pn-ragged", 2, 20, 9, 11, 37, 3, 2, 1, 1)], ids=lambda c: c.name)
def test_gemm_stage_with_nhwc_result(lib, cfg):
    x = uniform_int8(971, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(972, (cfg.K, cfg.C, cfg.R, cfg.S))
    want = layouts.unpack_nhwc(direct.conv2d_int8(x, w, cfg.stride, cfg.pad))
    for layout, cb in ((lib.LAYOUT_PACKED, 64), (lib.LAYOUT_IM2COL, 0)):
        xp = lib.im2col_int8(dev(x), cfg.R, cfg.S, cfg.stride, cfg.pad) if layout == lib.LAYOUT_IM2COL else lib.pack_layout(dev(x), cb, cfg.pad)
        wp = lib.pack_weights(dev(w), layout, cb)
        for split in (0, 2):
            out = torch.full(want.shape, -3, dtype=torch.int32, device=DEV)
            lib.conv2d_int8_packed_nhwc(cfg.dims(), layout, cb, xp, wp, out, split_k=split)
            assert np.array_equal(host(out), want), f"{lib.LAYOUT_NAMES[layout]} split {split}"


# ---- stencil unrolling from an NHWC source ---------------------------------------------------------------------
@pytest.mark.parametrize("cfg", [CONFIGS["C1"], CONFIGS["C2"], CONFIGS["C3"], CONFIGS["C4a"],
                                 ConvShape("in-ragged", 2, 37, 9, 11, 21, 3, 2, 2, 1), ConvShape("in-1ch", 1, 1, 20, 33, 8, 5, 4, 1, 2),
                                 ConvShape("in-48", 2, 48, 7, 6, 9, 3, 3, 1, 1)], ids=lambda c: c.name)
def test_im2col_from_nhwc(lib, cfg):
    x = uniform_int8(981, (cfg.N, cfg.C, cfg.H, cfg.W)); w = uniform_int8(982, (cfg.K, cfg.C, cfg.R, cfg.S))
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    A = lib.im2col_nhwc_int8(dev(xh), cfg.R, cfg.S, cfg.stride, cfg.pad)
    B = lib.pack_weights_rsc(dev(w))
    np.testing.assert_array_equal(host(A), layouts.im2col_nhwc(xh, cfg.R, cfg.S, cfg.stride, cfg.pad))
    np.testing.assert_array_equal(host(B), layouts.pack_weights_rsc(w))
    conv = direct.conv2d_int8(x, w, cfg.stride, cfg.pad)
    out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_IM2COL, 0, A, B, out)
    assert np.array_equal(host(out), conv)
    onh = torch.empty((cfg.N, cfg.P, cfg.Q, cfg.K), dtype=torch.int32, device=DEV)
    lib.conv2d_int8_packed_nhwc(cfg.dims(), lib.LAYOUT_IM2COL, 0, A, B, onh)     # NHWC in, NHWC out
    assert np.array_equal(host(onh), layouts.unpack_nhwc(conv))
