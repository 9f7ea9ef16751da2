"""GPU test of the entry point that allocates nothing (onnx_conv_fixed_scratch): called through
the raw C ABI on two convolutions in a row, the second smaller than the first, and compared with
onnx_conv using a caller-provided workspace of the same size (same split plan, so the bits must
agree) and with the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from util import REL_TOL, rel_err

pytestmark = pytest.mark.gpu


def _call(lib, fn, x, w, b, pads, strides, dil, group, res, act, y):
    from paper_2008_08272_amd import binding as B
    st = fn(B._ptr(x), B.dims(x.shape), B._ptr(w), B.dims(w.shape), B._ptr(b), B.dims(pads), B.dims(strides),
            B.dims(dil), int(group), B._ptr(res), int(act), B._ptr(y), B.dims(y.shape), B._stream(None))
    return st


def test_fixed_scratch_conv_two_calls_in_a_row():
    from paper_2008_08272_amd import binding as B
    assert torch.cuda.is_available(), "this test needs the GPU"
    lib = B.raw()
    rng = np.random.default_rng(2008)
    # few output tiles and a long K walk, so that both calls split K through the scratch:
    # 3x3 on 2x256x14x14 (LDS-patch kernel), then the smaller 1x1 on 1x1536x7x7 (contraction kernel)
    cases = [
        ((2, 256, 14, 14), (256, 256, 3, 3), (1, 1, 1, 1), (1, 1), (1, 1), 1, True),
        ((1, 1536, 7, 7), (128, 1536, 1, 1), (0, 0, 0, 0), (1, 1), (1, 1), 1, False),
    ]
    same_size_ws = torch.empty(B.CONV_FIXED_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    for i, (xs, ws_, pads, st, dl, g, with_res) in enumerate(cases):
        print("CASE fixed scratch", i, xs, ws_, flush=True)
        X = rng.uniform(-1, 1, xs).astype(np.float32)
        W = rng.uniform(-1, 1, ws_).astype(np.float32)
        Bv = rng.uniform(-1, 1, (ws_[0],)).astype(np.float32)
        yd = B.onnx_conv_infer(xs, ws_, pads, st, dl, g)
        R = rng.uniform(-1, 1, yd).astype(np.float32) if with_res else None
        ref = oracle.conv(X, W, Bv, pads, st, dl, g, residual=R, relu=True)
        x, w, b = (torch.from_numpy(a).cuda() for a in (X, W, Bv))
        r = torch.from_numpy(R).cuda() if with_res else None
        y_fixed = torch.full(yd, -7.0, dtype=torch.float32, device="cuda")
        y_ws = torch.full(yd, -9.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        # the entry point under test: no workspace set, nothing allocated by the call
        B.onnx_set_workspace(None)
        assert _call(lib, lib.onnx_conv_fixed_scratch, x, w, b, pads, st, dl, g, r, 1, y_fixed) == 0, B.onnx_last_error()
        launch = B.onnx_last_launch()
        assert "ksplit=1 " not in launch, launch            # the scratch really is in use
        # the existing entry point with a caller-provided workspace of the same size
        B.onnx_set_workspace(same_size_ws)
        assert _call(lib, lib.onnx_conv, x, w, b, pads, st, dl, g, r, 1, y_ws) == 0, B.onnx_last_error()
        assert B.onnx_last_launch() == launch
        B.onnx_set_workspace(None)
        torch.cuda.synchronize()
        got, want = y_fixed.cpu().numpy(), y_ws.cpu().numpy()
        assert np.array_equal(got, want), "fixed-scratch result differs from onnx_conv's"
        assert rel_err(got, ref) <= REL_TOL
    # a convolution above the stated maximum is refused, nothing written
    big = (B.CONV_FIXED_SCRATCH_MAX_OUTPUTS // (64 * 64)) + 1
    x = torch.zeros((1, 4, 64, 64), dtype=torch.float32, device="cuda")
    w = torch.zeros((big, 4, 1, 1), dtype=torch.float32, device="cuda")
    y = torch.full((1, big, 64, 64), 3.0, dtype=torch.float32, device="cuda")
    st = _call(lib, lib.onnx_conv_fixed_scratch, x, w, None, (0, 0, 0, 0), (1, 1), (1, 1), 1, None, 0, y)
    assert st == 5 and "exceed" in B.onnx_last_error()
    torch.cuda.synchronize()
    assert float(y.min()) == 3.0 and float(y.max()) == 3.0
