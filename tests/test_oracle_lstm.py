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


# ---- tile pattern on the fused weight (Section 3.2 on the LSTM of Section 7.2.3) ----

def _tile_synapse_mask(H, I, tr, tc, dp, b):
    return P.expand_tile_mask(P.tile_mask(4 * H, I + H, tr, tc, dp, b), 4 * H, I + H, tr, tc)


@pytest.mark.parametrize("tr,tc,dp,b", [(2, 3, 2, 1), (4, 2, 3, 3), (3, 3, 4, 2), (2, 2, 1, 1)])
def test_tile_pattern_lstm_is_textbook_lstm_on_masked_weights(tr, tc, dp, b):
    """A synapse mask is the ordinary LSTM with W o S for weights: torch.nn.LSTM forward, autograd backward
    (the gradient of a masked weight is the full gradient times the mask)."""
    T, B, I, H = 5, 3, 6, 4
    x, W, dh = _setup(3, T, B, I, H)
    S = _tile_synapse_mask(H, I, tr, tc, dp, b)
    assert 0 < S.sum() <= S.size and (dp == 1) == bool(S.all())
    fwd = L.lstm_forward_synapse(x, W, S, R.identity)
    bwd = L.lstm_backward_synapse(x, W, S, fwd, dh, R.identity)
    net = torch.nn.LSTM(I, H, bias=False).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.tensor(W * S)[:, :I])
        net.weight_hh_l0.copy_(torch.tensor(W * S)[:, I:])
    xt = torch.tensor(x, requires_grad=True)
    out, (hn, cn) = net(xt)
    (out * torch.tensor(dh)).sum().backward()
    assert np.allclose(fwd["h"], out.detach().numpy(), atol=1e-12)
    assert np.allclose(fwd["c"][-1], cn[0].detach().numpy(), atol=1e-12)
    assert np.allclose(bwd["dx"], xt.grad.numpy(), atol=1e-11)
    assert np.allclose(bwd["dW"][:, :I], net.weight_ih_l0.grad.numpy() * S[:, :I], atol=1e-11)
    assert np.allclose(bwd["dW"][:, I:], net.weight_hh_l0.grad.numpy() * S[:, I:], atol=1e-11)
    assert np.all(bwd["dW"][S == 0] == 0)


def test_dropped_synapses_have_no_influence():
    """Changing weights under dropped tiles changes nothing; changing a kept one does."""
    T, B, I, H = 4, 2, 5, 4
    x, W, dh = _setup(4, T, B, I, H)
    S = _tile_synapse_mask(H, I, 4, 3, 2, 2)
    ref = L.lstm_forward_synapse(x, W, S, R.identity)
    W2 = W + 7.0 * (1 - S)
    alt = L.lstm_forward_synapse(x, W2, S, R.identity)
    assert np.array_equal(ref["h"], alt["h"]) and np.array_equal(ref["gates"], alt["gates"])
    b1 = L.lstm_backward_synapse(x, W, S, ref, dh, R.identity)
    b2 = L.lstm_backward_synapse(x, W2, S, alt, dh, R.identity)
    assert np.array_equal(b1["dx"], b2["dx"]) and np.array_equal(b1["dW"], b2["dW"])
    r, c = np.argwhere(S == 1)[3]
    W3 = W.copy()
    W3[r, c] += 0.5
    assert not np.array_equal(L.lstm_forward_synapse(x, W3, S, R.identity)["h"], ref["h"])


def test_synapse_bptt_is_the_gradient():
    T, B, I, H = 3, 2, 4, 4
    x, W, dh = _setup(5, T, B, I, H)
    S = _tile_synapse_mask(H, I, 4, 4, 2, 1)
    fwd = L.lstm_forward_synapse(x, W, S, R.identity)
    bwd = L.lstm_backward_synapse(x, W, S, fwd, dh, R.identity)

    def loss(xv, Wv):
        return float(np.sum(dh * L.lstm_forward_synapse(xv, Wv, S, R.identity)["h"]))
    eps = 1e-6
    for idx in [(0, 0, 0), (1, 1, 3), (2, 0, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        assert abs((loss(xp, W) - loss(xm, W)) / (2 * eps) - bwd["dx"][idx]) < 1e-7
    kept = [tuple(rc) for rc in np.argwhere(S == 1)[::9]]
    dropped = [tuple(rc) for rc in np.argwhere(S == 0)[::17]]
    assert kept and dropped
    for idx in kept + dropped:
        Wp, Wm_ = W.copy(), W.copy()
        Wp[idx] += eps
        Wm_[idx] -= eps
        assert abs((loss(x, Wp) - loss(x, Wm_)) / (2 * eps) - bwd["dW"][idx]) < 1e-7


@pytest.mark.parametrize("dp,b", [(2, 1), (3, 2)])
def test_unit_mask_as_a_synapse_mask_gives_the_row_variant(dp, b):
    """A synapse mask that removes whole gate rows and recurrent columns of some units is the row variant:
    same h, c, dx, dW (a unit without incoming synapses has g = 0, so its cell and output stay 0)."""
    T, B, I, H = 4, 3, 5, 6
    x, W, dh = _setup(6, T, B, I, H)
    m = P.row_mask(H, dp, b)
    S = np.outer(np.tile(m, 4), np.concatenate([np.ones(I, np.uint8), m])).astype(np.uint8)
    fr = L.lstm_forward(x, W, m, R.identity)
    fs = L.lstm_forward_synapse(x, W, S, R.identity)
    assert np.allclose(fr["h"], fs["h"], atol=1e-14) and np.allclose(fr["c"], fs["c"], atol=1e-14)
    dhm = dh * m[None, None, :]          # the row variant ignores gradient arriving on dropped units
    br = L.lstm_backward(x, W, m, fr, dh, R.identity)
    bs = L.lstm_backward_synapse(x, W, S, fs, dhm, R.identity)
    assert np.allclose(br["dx"], bs["dx"], atol=1e-12) and np.allclose(br["dW"], bs["dW"], atol=1e-12)
