"""Pins for the oracle's LSTM under a hidden-unit row pattern (Section 7.2.3)."""
import numpy as np
import pytest
import torch

from oracle import lstm as L
from oracle import patterns as P
from oracle import rounding as R


def _setup(seed, T, B, I, H):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, B, I))
    W = rng.uniform(-0.5, 0.5, (4 * H, I + H))
    dh = rng.standard_normal((T, B, H))
    return x, W, dh


def test_rate_zero_is_textbook_lstm():
    """dp=1 must be the ordinary LSTM: check against torch.nn.LSTM (same i,f,g,o gate order)."""
    T, B, I, H = 5, 3, 6, 4
    x, W, dh = _setup(0, T, B, I, H)
    m = P.row_mask(H, 1, 1)
    fwd = L.lstm_forward(x, W, m, R.identity)
    bwd = L.lstm_backward(x, W, m, fwd, dh, R.identity)
    net = torch.nn.LSTM(I, H, bias=False).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.tensor(W[:, :I]))
        net.weight_hh_l0.copy_(torch.tensor(W[:, I:]))
    xt = torch.tensor(x, requires_grad=True)
    out, (hn, cn) = net(xt)
    (out * torch.tensor(dh)).sum().backward()
    assert np.allclose(fwd["h"], out.detach().numpy(), atol=1e-12)
    assert np.allclose(fwd["c"][-1], cn[0].detach().numpy(), atol=1e-12)
    assert np.allclose(bwd["dx"], xt.grad.numpy(), atol=1e-11)
    assert np.allclose(bwd["dW"][:, :I], net.weight_ih_l0.grad.numpy(), atol=1e-11)
    assert np.allclose(bwd["dW"][:, I:], net.weight_hh_l0.grad.numpy(), atol=1e-11)


@pytest.mark.parametrize("dp,b", [(2, 1), (2, 2), (3, 2)])
def test_masked_dense_equals_submodel(dp, b):
    """The masked layer equals a smaller textbook LSTM over the kept units only."""
    T, B, I, H = 4, 3, 5, 6
    x, W, dh = _setup(1, T, B, I, H)
    m = P.row_mask(H, dp, b)
    keep = P.keep_list(m)
    fwd = L.lstm_forward(x, W, m, R.identity)
    bwd = L.lstm_backward(x, W, m, fwd, dh, R.identity)
    rows = np.concatenate([g * H + keep for g in range(4)])
    cols = np.concatenate([np.arange(I), I + keep])
    Wc = W[np.ix_(rows, cols)]
    ones = np.ones(len(keep), np.uint8)
    fc = L.lstm_forward(x, Wc, ones, R.identity)
    bc = L.lstm_backward(x, Wc, ones, fc, dh[:, :, keep], R.identity)
    assert np.allclose(fwd["h"][:, :, keep], fc["h"], atol=1e-13)
    assert np.all(fwd["h"][:, :, m == 0] == 0) and np.all(fwd["c"][:, :, m == 0] == 0)
    assert np.allclose(bwd["dx"], bc["dx"], atol=1e-12)
    assert np.allclose(bwd["dW"][np.ix_(rows, cols)], bc["dW"], atol=1e-12)
    full = np.zeros_like(W)
    full[np.ix_(rows, cols)] = 1
    assert np.all(bwd["dW"][full == 0] == 0)


def test_bptt_is_the_gradient():
    T, B, I, H = 3, 2, 4, 4
    x, W, dh = _setup(2, T, B, I, H)
    m = P.row_mask(H, 2, 1)
    fwd = L.lstm_forward(x, W, m, R.identity)
    bwd = L.lstm_backward(x, W, m, fwd, dh, R.identity)

    def loss(xv, Wv):
        return float(np.sum(dh * L.lstm_forward(xv, Wv, m, R.identity)["h"]))
    eps = 1e-6
    for idx in [(0, 0, 0), (1, 1, 3), (2, 0, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        assert abs((loss(xp, W) - loss(xm, W)) / (2 * eps) - bwd["dx"][idx]) < 1e-7
    for idx in [(0, 0), (2, 5), (4, 6), (8, 1), (14, 4), (1, 0), (3, 5)]:
        Wp, Wm_ = W.copy(), W.copy()
        Wp[idx] += eps
        Wm_[idx] -= eps
        assert abs((loss(x, Wp) - loss(x, Wm_)) / (2 * eps) - bwd["dW"][idx]) < 1e-7
