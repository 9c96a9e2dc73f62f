"""ctypes binding for include/conv2d_int8.h: same names, argument marshalling only.

torch is used for device memory and streams, nothing else.  There is no CPU fallback:
if the HIP library has not been built, `load()` raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_OVERFLOW_RISK, ERR_WORKSPACE, ERR_DEVICE = range(6)
LAYOUT_AUTO, LAYOUT_PACKED, LAYOUT_IM2COL, LAYOUT_PAD_ONLY, LAYOUT_IMPLICIT, LAYOUT_IMAGE_PACK = range(6)
TILE_BAND = -2   # CONV_TILE_BAND
LAYOUT_NAMES = {LAYOUT_AUTO: "auto", LAYOUT_PACKED: "packed", LAYOUT_IM2COL: "im2col",
                LAYOUT_PAD_ONLY: "pad_only", LAYOUT_IMPLICIT: "implicit",
                LAYOUT_IMAGE_PACK: "image_pack"}

EXPORTS = [
    "conv2d_int8", "conv2d_int8_static", "conv2d_int8_nhwc", "unpack_nhwc_int32", "requant_int8", "requant_pack_layout", "conv2d_int8_ex", "conv2d_int8_workspace_bytes", "conv2d_int8_packed",
    "conv2d_int8_query_tiling", "conv2d_int8_num_tiles", "conv2d_int8_tile_info",
    "conv2d_int8_tile_applies", "conv2d_int8_tile_lds_bytes", "pack_layout", "pack_layout_bytes", "pack_layout_nhwc",
    "pack_weights", "pack_weights_depth", "pack_weights_bytes", "im2col_int8", "im2col_bytes",
    "image_pack_desc", "image_pack_bytes", "image_pack_weights_bytes", "image_pack_int8", "image_pack_weights",
    "conv2d_int8_packed_requant", "conv2d_int8_packed_nhwc", "mfma_probe_int8", "im2col_nhwc_int8", "pack_weights_rsc",
    "dilated_desc", "dilation_pack_bytes", "dilation_pack_int8", "dilation_unpack_int32",
    "conv2d_int8_dilated_workspace_bytes", "conv2d_int8_dilated",
    "conv2d_int8_dilated_direct_workspace_bytes", "conv2d_int8_dilated_direct",
    "gemm_int8_nt", "select_layout", "select_layout_weighted", "layout_overheads",
    "conv_status_string",
]


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")]


class ConvError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def load(path: str | None = None):
    """Load the built library (never builds; never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or _build.LIB
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python -m paper_2104_04731_amd.build` "
                           "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(path)
    i, vp, sz, dbl = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double
    dp, ip = ctypes.POINTER(ConvDesc), ctypes.POINTER(ctypes.c_int)
    sig = {
        "conv2d_int8": (i, [i] * 9 + [vp, vp, vp, vp]),
        "conv2d_int8_static": (i, [i] * 9 + [vp, vp, vp, vp]),
        "conv2d_int8_nhwc": (i, [i] * 9 + [vp, vp, vp, vp]),
        "unpack_nhwc_int32": (i, [i] * 4 + [vp, vp, vp]),
        "requant_int8": (i, [ctypes.c_longlong, vp, vp, i, i, vp]),
        "requant_pack_layout": (i, [i] * 8 + [vp, vp, vp]),
        "conv2d_int8_ex": (i, [dp, i, i, vp, vp, i, vp, vp, sz, vp]),
        "conv2d_int8_workspace_bytes": (sz, [dp, i, i, i]),
        "conv2d_int8_packed": (i, [dp, i, i, vp, vp, vp, i, i, vp]),
        "conv2d_int8_query_tiling": (i, [dp, i, i, ip, ip]),
        "conv2d_int8_tile_applies": (i, [dp, i, i, i, i]),
        "conv2d_int8_tile_lds_bytes": (sz, [dp, i, i, i, i]),
        "conv2d_int8_num_tiles": (i, []),
        "conv2d_int8_tile_info": (i, [i, ip, ip, ip, ip]),
        "pack_layout": (i, [i] * 6 + [vp, vp, vp]),
        "pack_layout_bytes": (sz, [i] * 6),
        "pack_layout_nhwc": (i, [i] * 6 + [vp, vp, vp]),
        "pack_weights": (i, [i] * 6 + [vp, vp, vp]),
        "pack_weights_depth": (i, [i] * 5),
        "pack_weights_bytes": (sz, [i] * 6),
        "im2col_int8": (i, [i] * 9 + [vp, vp, vp]),
        "im2col_bytes": (sz, [i] * 9),
        "im2col_nhwc_int8": (i, [i] * 9 + [vp, vp, vp]),
        "pack_weights_rsc": (i, [i] * 4 + [vp, vp, vp]),
        "image_pack_desc": (i, [dp, dp]),
        "image_pack_bytes": (sz, [dp]),
        "image_pack_weights_bytes": (sz, [dp]),
        "image_pack_int8": (i, [dp, vp, vp, vp]),
        "image_pack_weights": (i, [dp, vp, vp, vp]),
        "conv2d_int8_packed_requant": (i, [dp, i, i, vp, vp, vp, i, i, i, i, vp]),
        "conv2d_int8_packed_nhwc": (i, [dp, i, i, vp, vp, vp, i, i, vp]),
        "dilated_desc": (i, [dp, i, dp]),
        "dilation_pack_bytes": (sz, [dp, i]),
        "dilation_pack_int8": (i, [dp, i, vp, vp, vp]),
        "dilation_unpack_int32": (i, [dp, i, vp, vp, vp]),
        "conv2d_int8_dilated_workspace_bytes": (sz, [dp, i, i, i]),
        "conv2d_int8_dilated": (i, [dp, i, i, i, vp, vp, vp, vp, sz, vp]),
        "mfma_probe_int8": (i, [i, i, vp, vp]),
        "conv2d_int8_dilated_direct_workspace_bytes": (sz, [dp, i, i]),
        "conv2d_int8_dilated_direct": (i, [dp, i, i, vp, vp, vp, vp, sz, vp]),
        "gemm_int8_nt": (i, [i, i, i, vp, vp, vp, vp]),
        "select_layout": (i, [dp, ip, ip, ctypes.POINTER(dbl)]),
        "select_layout_weighted": (i, [dp, dbl, dbl, ip, ip, ctypes.POINTER(dbl)]),
        "layout_overheads": (i, [dp, i, i] + [ctypes.POINTER(ctypes.c_int64)] * 3),
        "conv_status_string": (ctypes.c_char_p, [i]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().conv_status_string(int(status)).decode()


def _check(status, what):
    if status != OK:
        raise ConvError(status, what)


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t: torch.Tensor):
    return ctypes.c_void_p(t.data_ptr())


def _desc(N, C, H, W, K, R, S, stride, pad):
    return ConvDesc(N, C, H, W, K, R, S, stride, pad)


def out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def _require(t, dtype, what):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what} must be a contiguous {dtype} CUDA tensor")


# ---- one-shot -------------------------------------------------------------------------------
def conv2d_int8(x: torch.Tensor, w: torch.Tensor, stride: int, pad: int, out=None, stream=None):
    _require(x, torch.int8, "input"); _require(w, torch.int8, "weights")
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = out_hw(H, W, R, S, stride, pad)
    if out is None:
        out = torch.empty((N, K, max(P, 0), max(Q, 0)), dtype=torch.int32, device=x.device)
    _check(load().conv2d_int8(N, C, H, W, K, R, S, stride, pad, _ptr(x), _ptr(w), _ptr(out),
                              _stream(stream)), "conv2d_int8")
    return out


STATIC_WORKSPACE_BYTES = 8 << 20


def conv2d_int8_static(x: torch.Tensor, w: torch.Tensor, stride: int, pad: int, out: torch.Tensor, stream=None):
    """conv2d_int8 through the library's fixed device array: the call allocates nothing (`out` is the caller's)."""
    _require(x, torch.int8, "input"); _require(w, torch.int8, "weights"); _require(out, torch.int32, "output")
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    _check(load().conv2d_int8_static(N, C, H, W, K, R, S, stride, pad, _ptr(x), _ptr(w), _ptr(out),
                                     _stream(stream)), "conv2d_int8_static")
    return out


def conv2d_int8_nhwc(x: torch.Tensor, w: torch.Tensor, stride: int, pad: int, out=None, stream=None):
    """x: [N, H, W, C] int8, w: KCRS int8 -> [N, P, Q, K] int32."""
    _require(x, torch.int8, "input"); _require(w, torch.int8, "weights")
    N, H, W, C = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = out_hw(H, W, R, S, stride, pad)
    if out is None:
        out = torch.empty((N, max(P, 0), max(Q, 0), K), dtype=torch.int32, device=x.device)
    _check(load().conv2d_int8_nhwc(N, C, H, W, K, R, S, stride, pad, _ptr(x), _ptr(w), _ptr(out),
                                   _stream(stream)), "conv2d_int8_nhwc")
    return out


def unpack_nhwc_int32(x: torch.Tensor, out=None, stream=None):
    """[N, K, P, Q] int32 -> [N, P, Q, K] int32."""
    _require(x, torch.int32, "NKPQ tensor")
    N, K, P, Q = x.shape
    if out is None:
        out = torch.empty((N, P, Q, K), dtype=torch.int32, device=x.device)
    _check(load().unpack_nhwc_int32(N, K, P, Q, _ptr(x), _ptr(out), _stream(stream)), "unpack_nhwc_int32")
    return out


def requant_int8(x: torch.Tensor, shift: int, relu: bool, out=None, stream=None):
    """int32 tensor -> int8 tensor of the same shape: clip(relu(floor(x / 2^shift + 1/2)))."""
    _require(x, torch.int32, "accumulator tensor")
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(load().requant_int8(x.numel(), _ptr(x), _ptr(out), shift, int(relu), _stream(stream)), "requant_int8")
    return out


def requant_pack_layout(x: torch.Tensor, cb: int, pad: int, shift: int, relu: bool, out=None, stream=None):
    """[N, K, P, Q] int32 -> [N, ceil(K/cb), P+2pad, Q+2pad, cb] int8: activation + the next layer's blocking."""
    _require(x, torch.int32, "accumulator tensor")
    N, K, P, Q = x.shape
    if out is None:
        if cb % 16:
            _check(ERR_UNSUPPORTED, "requant_pack_layout")
        out = torch.empty((N, (K + cb - 1) // cb, P + 2 * pad, Q + 2 * pad, cb), dtype=torch.int8, device=x.device)
    _check(load().requant_pack_layout(N, K, P, Q, cb, pad, shift, int(relu), _ptr(x), _ptr(out), _stream(stream)),
           "requant_pack_layout")
    return out


def conv2d_int8_workspace_bytes(dims, layout=LAYOUT_AUTO, cb=0, wt_is_packed=False) -> int:
    d = _desc(*dims)
    return int(load().conv2d_int8_workspace_bytes(ctypes.byref(d), layout, cb, int(wt_is_packed)))


def conv2d_int8_ex(dims, layout, cb, x, w, out, workspace, wt_is_packed=False, stream=None):
    d = _desc(*dims)
    ws_ptr = _ptr(workspace) if workspace is not None else ctypes.c_void_p(0)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().conv2d_int8_ex(ctypes.byref(d), layout, cb, _ptr(x), _ptr(w), int(wt_is_packed),
                                 _ptr(out), ws_ptr, ws_bytes, _stream(stream)), "conv2d_int8_ex")
    return out


def conv2d_int8_packed(dims, layout, cb, x_packed, w_packed, out, tile=-1, split_k=0, stream=None):
    d = _desc(*dims)
    _check(load().conv2d_int8_packed(ctypes.byref(d), layout, cb, _ptr(x_packed), _ptr(w_packed),
                                     _ptr(out), tile, split_k, _stream(stream)), "conv2d_int8_packed")
    return out


def conv2d_int8_packed_nhwc(dims, layout, cb, x_packed, w_packed, out, tile=-1, split_k=0, stream=None):
    """GEMM stage writing int32 [N][P][Q][K]."""
    d = _desc(*dims)
    _check(load().conv2d_int8_packed_nhwc(ctypes.byref(d), layout, cb, _ptr(x_packed), _ptr(w_packed),
                                          _ptr(out), tile, split_k, _stream(stream)), "conv2d_int8_packed_nhwc")
    return out


def tile_applies(dims, layout, cb, tile, split_k=1):
    """True if conv2d_int8_packed would accept this forced tile and depth split."""
    d = _desc(*dims)
    return load().conv2d_int8_tile_applies(ctypes.byref(d), layout, cb, tile, split_k) == OK


def tile_lds_bytes(dims, layout, cb, tile, split_k=1) -> int:
    d = _desc(*dims)
    return int(load().conv2d_int8_tile_lds_bytes(ctypes.byref(d), layout, cb, tile, split_k))


def query_tiling(dims, layout, cb):
    d = _desc(*dims)
    t, s = ctypes.c_int(), ctypes.c_int()
    _check(load().conv2d_int8_query_tiling(ctypes.byref(d), layout, cb, ctypes.byref(t), ctypes.byref(s)),
           "conv2d_int8_query_tiling")
    return t.value, s.value


def num_tiles() -> int:
    return load().conv2d_int8_num_tiles()


def tile_info(tile: int):
    r, c, t, k = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(load().conv2d_int8_tile_info(tile, ctypes.byref(r), ctypes.byref(c), ctypes.byref(t),
                                        ctypes.byref(k)), "conv2d_int8_tile_info")
    return r.value, c.value, t.value, k.value


# ---- layout rewrites ------------------------------------------------------------------------
def pack_layout_bytes(N, C, H, W, cb, pad) -> int:
    return int(load().pack_layout_bytes(N, C, H, W, cb, pad))


def pack_layout(x: torch.Tensor, cb: int, pad: int, out=None, stream=None):
    _require(x, torch.int8, "input")
    N, C, H, W = x.shape
    nbytes = pack_layout_bytes(N, C, H, W, cb, pad)
    if out is None:
        if nbytes == 0:
            _check(ERR_UNSUPPORTED, "pack_layout")
        out = torch.empty((N, (C + cb - 1) // cb, H + 2 * pad, W + 2 * pad, cb), dtype=torch.int8,
                          device=x.device)
    _check(load().pack_layout(N, C, H, W, cb, pad, _ptr(x), _ptr(out), _stream(stream)), "pack_layout")
    return out


def pack_layout_nhwc(x: torch.Tensor, cb: int, pad: int, out=None, stream=None):
    """x: [N, H, W, C] int8."""
    _require(x, torch.int8, "input")
    N, H, W, C = x.shape
    if out is None:
        if pack_layout_bytes(N, C, H, W, cb, pad) == 0 or cb % 16:
            _check(ERR_UNSUPPORTED, "pack_layout_nhwc")
        out = torch.empty((N, (C + cb - 1) // cb, H + 2 * pad, W + 2 * pad, cb), dtype=torch.int8,
                          device=x.device)
    _check(load().pack_layout_nhwc(N, C, H, W, cb, pad, _ptr(x), _ptr(out), _stream(stream)), "pack_layout_nhwc")
    return out


def pack_weights_depth(C, R, S, layout, cb) -> int:
    return int(load().pack_weights_depth(C, R, S, layout, cb))


def pack_weights_bytes(K, C, R, S, layout, cb) -> int:
    return int(load().pack_weights_bytes(K, C, R, S, layout, cb))


def pack_weights(w: torch.Tensor, layout: int, cb: int, out=None, stream=None):
    _require(w, torch.int8, "weights")
    K, C, R, S = w.shape
    if out is None:
        depth = pack_weights_depth(C, R, S, layout, cb)
        if depth == 0:
            _check(ERR_UNSUPPORTED, "pack_weights")
        out = torch.empty((K, depth), dtype=torch.int8, device=w.device)
    _check(load().pack_weights(K, C, R, S, layout, cb, _ptr(w), _ptr(out), _stream(stream)),
           "pack_weights")
    return out


def im2col_bytes(N, C, H, W, R, S, stride, pad, kg_pad) -> int:
    return int(load().im2col_bytes(N, C, H, W, R, S, stride, pad, kg_pad))


def im2col_int8(x: torch.Tensor, R, S, stride, pad, kg_pad=None, out=None, stream=None):
    _require(x, torch.int8, "input")
    N, C, H, W = x.shape
    if kg_pad is None:
        kg_pad = (C * R * S + 63) // 64 * 64
    if out is None:
        P, Q = out_hw(H, W, R, S, stride, pad)
        out = torch.empty((N * max(P, 0) * max(Q, 0), kg_pad), dtype=torch.int8, device=x.device)
    _check(load().im2col_int8(N, C, H, W, R, S, stride, pad, kg_pad, _ptr(x), _ptr(out),
                              _stream(stream)), "im2col_int8")
    return out


def im2col_nhwc_int8(xh: torch.Tensor, R, S, stride, pad, kg_pad=None, out=None, stream=None):
    """xh: [N, H, W, C] int8 -> [N*P*Q, kg_pad], depth index (r*S + s)*C + c."""
    _require(xh, torch.int8, "input")
    N, H, W, C = xh.shape
    if kg_pad is None:
        kg_pad = -(-C * R * S // 64) * 64
    if out is None:
        P, Q = out_hw(H, W, R, S, stride, pad)
        out = torch.empty((N * max(P, 0) * max(Q, 0), kg_pad), dtype=torch.int8, device=xh.device)
    _check(load().im2col_nhwc_int8(N, C, H, W, R, S, stride, pad, kg_pad, _ptr(xh), _ptr(out), _stream(stream)),
           "im2col_nhwc_int8")
    return out


def pack_weights_rsc(w: torch.Tensor, out=None, stream=None):
    """KCRS int8 -> [K, ceil(C*R*S, 64)] in the depth order of im2col_nhwc_int8."""
    _require(w, torch.int8, "weights")
    K, C, R, S = w.shape
    if out is None:
        out = torch.empty((K, -(-C * R * S // 64) * 64), dtype=torch.int8, device=w.device)
    _check(load().pack_weights_rsc(K, C, R, S, _ptr(w), _ptr(out), _stream(stream)), "pack_weights_rsc")
    return out


def image_pack_desc(dims):
    """The stride-1, pad-0 problem (N, C2, H2, W2, K, R2, S2, 1, 0) an image-packed convolution turns into."""
    d, d2 = _desc(*dims), ConvDesc()
    _check(load().image_pack_desc(ctypes.byref(d), ctypes.byref(d2)), "image_pack_desc")
    return tuple(getattr(d2, f) for f, _ in ConvDesc._fields_)


def image_pack_int8(dims, x: torch.Tensor, out=None, stream=None):
    _require(x, torch.int8, "input")
    d = _desc(*dims)
    if out is None:
        N, C2, H2, W2 = image_pack_desc(dims)[:4]
        out = torch.empty((N, C2, H2, W2), dtype=torch.int8, device=x.device)
    _check(load().image_pack_int8(ctypes.byref(d), _ptr(x), _ptr(out), _stream(stream)), "image_pack_int8")
    return out


def image_pack_weights(dims, w: torch.Tensor, out=None, stream=None):
    _require(w, torch.int8, "weights")
    d = _desc(*dims)
    if out is None:
        _, C2, _, _, K, R2, S2, _, _ = image_pack_desc(dims)
        out = torch.empty((K, C2, R2, S2), dtype=torch.int8, device=w.device)
    _check(load().image_pack_weights(ctypes.byref(d), _ptr(w), _ptr(out), _stream(stream)), "image_pack_weights")
    return out


def conv2d_int8_packed_requant(dims, layout, cb, x_packed: torch.Tensor, w_packed: torch.Tensor, out_cb, out_pad, shift, relu,
                               out=None, stream=None):
    """GEMM stage with the activation in its epilogue: returns the next layer's blocked int8 input."""
    N, C, H, W, K, R, S, stride, pad = dims
    if out is None:
        P, Q = out_hw(H, W, R, S, stride, pad)
        out = torch.empty((N, -(-K // out_cb), P + 2 * out_pad, Q + 2 * out_pad, out_cb), dtype=torch.int8, device=x_packed.device)
    _check(load().conv2d_int8_packed_requant(ctypes.byref(_desc(*dims)), int(layout), int(cb), _ptr(x_packed), _ptr(w_packed),
                                             _ptr(out), int(out_cb), int(out_pad), int(shift), int(bool(relu)),
                                             _stream(stream)), "conv2d_int8_packed_requant")
    return out


def dilated_desc(dims, dilation):
    """The dense stride-1, pad-0 problem (N*d*d, C, H2, W2, K, R, S, 1, 0) a dilated convolution turns into."""
    d, d2 = _desc(*dims), ConvDesc()
    _check(load().dilated_desc(ctypes.byref(d), int(dilation), ctypes.byref(d2)), "dilated_desc")
    return tuple(getattr(d2, f) for f, _ in ConvDesc._fields_)


def dilated_out_hw(dims, dilation):
    N, C, H, W, K, R, S, stride, pad = dims
    return H + 2 * pad - dilation * (R - 1), W + 2 * pad - dilation * (S - 1)


def dilation_pack_int8(dims, dilation, x: torch.Tensor, out=None, stream=None):
    _require(x, torch.int8, "input")
    d = _desc(*dims)
    if out is None:
        N2, C, H2, W2 = dilated_desc(dims, dilation)[:4]
        out = torch.empty((N2, C, H2, W2), dtype=torch.int8, device=x.device)
    _check(load().dilation_pack_int8(ctypes.byref(d), int(dilation), _ptr(x), _ptr(out), _stream(stream)),
           "dilation_pack_int8")
    return out


def dilation_unpack_int32(dims, dilation, o2: torch.Tensor, out=None, stream=None):
    _require(o2, torch.int32, "sub-image results")
    d = _desc(*dims)
    if out is None:
        P, Q = dilated_out_hw(dims, dilation)
        out = torch.empty((dims[0], dims[4], P, Q), dtype=torch.int32, device=o2.device)
    _check(load().dilation_unpack_int32(ctypes.byref(d), int(dilation), _ptr(o2), _ptr(out), _stream(stream)),
           "dilation_unpack_int32")
    return out


def conv2d_int8_dilated_workspace_bytes(dims, dilation, layout=LAYOUT_AUTO, cb=0) -> int:
    return int(load().conv2d_int8_dilated_workspace_bytes(ctypes.byref(_desc(*dims)), int(dilation), int(layout), int(cb)))


def conv2d_int8_dilated(dims, dilation, x: torch.Tensor, w: torch.Tensor, layout=LAYOUT_AUTO, cb=0, out=None,
                        workspace=None, stream=None):
    """Stride-1 convolution with dilation >= 2: sub-images into the batch, dense convolution, interleave."""
    _require(x, torch.int8, "input"); _require(w, torch.int8, "weights")
    d = _desc(*dims)
    if out is None:
        P, Q = dilated_out_hw(dims, dilation)
        out = torch.empty((dims[0], dims[4], max(P, 0), max(Q, 0)), dtype=torch.int32, device=x.device)
    if workspace is None:
        need = conv2d_int8_dilated_workspace_bytes(dims, dilation, layout, cb)
        workspace = torch.empty(need + 256, dtype=torch.int8, device=x.device)
        workspace = workspace[(-workspace.data_ptr()) % 256:]
    _check(load().conv2d_int8_dilated(ctypes.byref(d), int(dilation), int(layout), int(cb), _ptr(x), _ptr(w), _ptr(out),
                                      _ptr(workspace), workspace.numel(), _stream(stream)), "conv2d_int8_dilated")
    return out


def conv2d_int8_dilated_direct(dims, dilation, x: torch.Tensor, w: torch.Tensor, cb=0, out=None, workspace=None, stream=None):
    """Dilated convolution (any stride) with the dilation as an address multiplier of the GEMM stage."""
    _require(x, torch.int8, "input"); _require(w, torch.int8, "weights")
    N, C, H, W, K, R, S, stride, pad = dims
    d = _desc(*dims)
    if out is None:
        P = (H + 2 * pad - dilation * (R - 1) - 1) // stride + 1
        Q = (W + 2 * pad - dilation * (S - 1) - 1) // stride + 1
        out = torch.empty((N, K, max(P, 0), max(Q, 0)), dtype=torch.int32, device=x.device)
    if workspace is None:
        need = int(load().conv2d_int8_dilated_direct_workspace_bytes(ctypes.byref(d), int(dilation), int(cb)))
        workspace = torch.empty(need + 256, dtype=torch.int8, device=x.device)
        workspace = workspace[(-workspace.data_ptr()) % 256:]
    _check(load().conv2d_int8_dilated_direct(ctypes.byref(d), int(dilation), int(cb), _ptr(x), _ptr(w), _ptr(out),
                                             _ptr(workspace), workspace.numel(), _stream(stream)), "conv2d_int8_dilated_direct")
    return out


def mfma_probe_int8(blocks: int, iters: int, out=None, stream=None, device="cuda:0"):
    """Register-resident MFMA loop; returns (checksums, operations issued)."""
    if out is None:
        out = torch.empty(blocks * 256, dtype=torch.int32, device=device)
    _check(load().mfma_probe_int8(int(blocks), int(iters), _ptr(out), _stream(stream)), "mfma_probe_int8")
    return out, 2 * 32768 * 16 * int(iters) * int(blocks)


def gemm_int8_nt(A: torch.Tensor, B: torch.Tensor, out=None, stream=None):
    _require(A, torch.int8, "A"); _require(B, torch.int8, "B")
    X, Z = A.shape
    Y, Z2 = B.shape
    if Z != Z2:
        raise ValueError("depth mismatch")
    if out is None:
        out = torch.empty((X, Y), dtype=torch.int32, device=A.device)
    _check(load().gemm_int8_nt(X, Y, Z, _ptr(A), _ptr(B), _ptr(out), _stream(stream)), "gemm_int8_nt")
    return out


# ---- selection (host only) --------------------------------------------------------------------
def select_layout(dims, w_mac=None, w_data=None):
    d = _desc(*dims)
    lay, cb, sc = ctypes.c_int(), ctypes.c_int(), ctypes.c_double()
    if w_mac is None:
        st = load().select_layout(ctypes.byref(d), ctypes.byref(lay), ctypes.byref(cb), ctypes.byref(sc))
    else:
        st = load().select_layout_weighted(ctypes.byref(d), w_mac, w_data, ctypes.byref(lay),
                                           ctypes.byref(cb), ctypes.byref(sc))
    _check(st, "select_layout")
    return lay.value, cb.value, sc.value


def layout_applies(dims, layout, cb=0) -> bool:
    """Whether the library has this layout for this problem (layout_overheads is the domain query)."""
    d = _desc(*dims)
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    st = load().layout_overheads(ctypes.byref(d), layout, cb, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if st not in (OK, ERR_UNSUPPORTED):
        raise ConvError(st, "layout_overheads")
    return st == OK


def layout_overheads(dims, layout, cb):
    d = _desc(*dims)
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(load().layout_overheads(ctypes.byref(d), layout, cb, ctypes.byref(a), ctypes.byref(b),
                                   ctypes.byref(c)), "layout_overheads")
    return a.value, b.value, c.value
