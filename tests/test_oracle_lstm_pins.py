"""Pins for the LSTM oracle: a hand-worked single step, structural identities, and torch's CPU LSTM in
float64 (an independent implementation; its gate order i, f, g, o is permuted into ONNX's i, o, f, c)."""
import math

import numpy as np
import pytest

from oracle.lstm import lstm


def sig(v):
    return 1.0 / (1.0 + math.exp(-v))


def test_single_step_by_hand():
    # H = 1, input = 1, batch = 1: W rows (i, o, f, c) = 1, 2, 3, 4; R = 0.5 each; biases Wb = 0.1 k, Rb = 0.01 k
    X = np.array([[[0.5]]], np.float32)
    W = np.array([[[1.0], [2.0], [3.0], [4.0]]], np.float32)
    R = np.full((1, 4, 1), 0.5, np.float32)
    B = np.array([[0.1, 0.2, 0.3, 0.4, 0.01, 0.02, 0.03, 0.04]], np.float32)
    h0 = np.array([[[0.25]]], np.float32)
    c0 = np.array([[[-1.0]]], np.float32)
    f32 = lambda v: float(np.float32(v))
    pre = [f32(w) * 0.5 + 0.5 * 0.25 + f32(wb) + f32(rb) for w, wb, rb in
           zip((1, 2, 3, 4), (0.1, 0.2, 0.3, 0.4), (0.01, 0.02, 0.03, 0.04))]
    i, o, f, g = sig(pre[0]), sig(pre[1]), sig(pre[2]), math.tanh(pre[3])
    c = f * -1.0 + i * g
    h = o * math.tanh(c)
    Y, Yh, Yc = lstm(X, W, R, B, h0, c0)
    assert Y.shape == (1, 1, 1, 1)
    assert abs(Y[0, 0, 0, 0] - h) < 1e-15 and abs(Yh[0, 0, 0] - h) < 1e-15 and abs(Yc[0, 0, 0] - c) < 1e-15


def test_structure():
    rng = np.random.default_rng(3)
    seq, batch, inp, H = 5, 3, 4, 6
    X = rng.standard_normal((seq, batch, inp)).astype(np.float32)
    W = rng.standard_normal((2, 4 * H, inp)).astype(np.float32) * 0.4
    R = rng.standard_normal((2, 4 * H, H)).astype(np.float32) * 0.4
    B = rng.standard_normal((2, 8 * H)).astype(np.float32) * 0.2
    Yf, hf, cf = lstm(X, W[:1], R[:1], B[:1])
    Yr, hr, cr = lstm(X, W[1:], R[1:], B[1:], direction="reverse")
    Yb, hb, cb = lstm(X, W, R, B, direction="bidirectional")
    assert np.array_equal(Yb[:, 0], Yf[:, 0]) and np.array_equal(Yb[:, 1], Yr[:, 0])      # directions are independent
    assert np.array_equal(hb[0], hf[0]) and np.array_equal(cb[1], cr[0])
    assert np.array_equal(hf[0], Yf[-1, 0]) and np.array_equal(hr[0], Yr[0, 0])            # last step of each direction
    # reverse = forward on the time-reversed sequence
    Y2, h2, c2 = lstm(X[::-1], W[1:], R[1:], B[1:])
    assert np.allclose(Y2[::-1], Yr, rtol=1e-13, atol=1e-15) and np.allclose(h2, hr, rtol=1e-13, atol=1e-15)
    # running the second half from the first half's state equals running the whole sequence
    Ya, ha, ca = lstm(X[:2], W[:1], R[:1], B[:1])
    Yb2, _, _ = lstm(X[2:], W[:1], R[:1], B[:1], ha.astype(np.float64), ca.astype(np.float64))
    # (states are handed over in double here, so the results agree to rounding of the conversion)
    assert np.allclose(Yb2, Yf[2:], rtol=1e-6, atol=1e-7)
    # batch rows are independent
    Y1, _, _ = lstm(X[:, 1:2], W[:1], R[:1], B[:1])
    assert np.allclose(Y1[:, 0, 0], Yf[:, 0, 1], rtol=1e-13, atol=1e-15)      # (BLAS may sum in another order)
    # |h| < 1, and zero weights give h = sigmoid(0) * tanh(sigmoid(0) * tanh(0)) = 0
    assert np.abs(Yf).max() < 1.0
    Z, _, _ = lstm(X, np.zeros_like(W[:1]), np.zeros_like(R[:1]))
    assert np.array_equal(Z, np.zeros_like(Z))


@pytest.mark.parametrize("direction", ["forward", "reverse", "bidirectional"])
def test_against_torch_float64(direction):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    seq, batch, inp, H = 7, 3, 5, 4
    dirs = 2 if direction == "bidirectional" else 1
    X = rng.standard_normal((seq, batch, inp)).astype(np.float32)
    W = (rng.standard_normal((dirs, 4 * H, inp)) * 0.5).astype(np.float32)
    R = (rng.standard_normal((dirs, 4 * H, H)) * 0.5).astype(np.float32)
    B = (rng.standard_normal((dirs, 8 * H)) * 0.3).astype(np.float32)
    h0 = (rng.standard_normal((dirs, batch, H)) * 0.5).astype(np.float32)
    c0 = (rng.standard_normal((dirs, batch, H)) * 0.5).astype(np.float32)
    Y, Yh, Yc = lstm(X, W, R, B, h0, c0, direction)
    net = torch.nn.LSTM(inp, H, bidirectional=dirs == 2).double()
    perm = np.concatenate([np.arange(0, H), np.arange(2 * H, 3 * H), np.arange(3 * H, 4 * H), np.arange(H, 2 * H)])  # ONNX iofc -> torch ifgo
    xin = X if direction != "reverse" else X[::-1].copy()
    with torch.no_grad():
        for d in range(dirs):
            sfx = "_reverse" if d == 1 else ""
            getattr(net, "weight_ih_l0" + sfx).copy_(torch.from_numpy(W[d][perm]).double())
            getattr(net, "weight_hh_l0" + sfx).copy_(torch.from_numpy(R[d][perm]).double())
            getattr(net, "bias_ih_l0" + sfx).copy_(torch.from_numpy(B[d][:4 * H][perm]).double())
            getattr(net, "bias_hh_l0" + sfx).copy_(torch.from_numpy(B[d][4 * H:][perm]).double())
        out, (hn, cn) = net(torch.from_numpy(xin).double(), (torch.from_numpy(h0).double(), torch.from_numpy(c0).double()))
    out = out.numpy().reshape(seq, batch, dirs, H).transpose(0, 2, 1, 3)
    if direction == "reverse":
        out = out[::-1]
    assert np.allclose(Y, out, rtol=1e-12, atol=1e-13)
    assert np.allclose(Yh, hn.numpy(), rtol=1e-12, atol=1e-13) and np.allclose(Yc, cn.numpy(), rtol=1e-12, atol=1e-13)
