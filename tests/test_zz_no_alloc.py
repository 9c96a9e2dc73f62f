"""The entry point that allocates nothing (conv2d_int8_static), through the C-ABI, against the one-shot
entry point it is a variant of: bit-exact, on two calls in a row, the second on a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import direct
from paper_2104_04731_amd.inputs import CONFIGS, ConvShape

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_both(lib, cfg, x, w):
    """(result of conv2d_int8_static, result of conv2d_int8) on the same device tensors, raw C-ABI calls."""
    raw = lib.load()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    outs = []
    for fn in (raw.conv2d_int8_static, raw.conv2d_int8):
        out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), -7, dtype=torch.int32, device=DEV)
        rc = fn(cfg.N, cfg.C, cfg.H, cfg.W, cfg.K, cfg.R, cfg.S, cfg.stride, cfg.pad,
                ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w.data_ptr()), ctypes.c_void_p(out.data_ptr()), st)
        assert rc == lib.OK, (fn.__name__, lib.status_string(rc))
        outs.append(out)
    torch.cuda.synchronize()
    return outs[0].cpu().numpy(), outs[1].cpu().numpy()


def test_static_workspace_two_calls_second_smaller(lib):
    # channel blocking both times (the layouts that use the workspace): 1.7 MB of it, then 0.25 MB of the same
    # bytes; then a depth-split problem (its output is cleared by a kernel), then a layout that needs none
    big, small = CONFIGS["C4a"], CONFIGS["C2"]
    deep = ConvShape("deep-small", 1, 256, 7, 7, 64, 3, 3, 1, 1)
    for cfg in (big, small, deep, CONFIGS["C3"], big):
        assert 0 <= lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_AUTO, 0) <= lib.STATIC_WORKSPACE_BYTES
        x, w = cfg.make()
        dx, dw = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
        got, ref = _run_both(lib, cfg, dx, dw)
        assert np.array_equal(got, ref), cfg.name
        assert np.array_equal(got, direct.conv2d_int8(x, w, cfg.stride, cfg.pad)), cfg.name


def test_static_workspace_refuses_what_does_not_fit(lib):
    cfg = CONFIGS["C2"].scaled(64)          # 13.8 MB of rewritten input
    assert lib.conv2d_int8_workspace_bytes(cfg.dims(), lib.LAYOUT_AUTO, 0) > lib.STATIC_WORKSPACE_BYTES
    x = torch.zeros((cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=DEV)
    w = torch.zeros((cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=DEV)
    out = torch.full((cfg.N, cfg.K, cfg.P, cfg.Q), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(lib.ConvError) as e:
        lib.conv2d_int8_static(x, w, cfg.stride, cfg.pad, out)
    assert e.value.status == lib.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert int((out != -7).sum()) == 0      # nothing was enqueued
