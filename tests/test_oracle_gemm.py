"""Pins for the oracle's masked GEMMs (Sections 3.1, 3.2) and the MLP chain."""
import numpy as np
import pytest

from oracle import gemm as G
from oracle import patterns as P
from oracle import rounding as R


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _brute_fwd(X, W, MW, m_out, alpha):
    B, I = X.shape
    O = W.shape[0]
    Y = np.zeros((B, O))
    for r in range(B):
        for o in range(O):
            if not m_out[o]:
                continue
            acc = 0.0
            for i in range(I):
                if MW[o, i]:
                    acc += X[r, i] * W[o, i]
            Y[r, o] = alpha * acc
    return Y


def test_rate_zero_is_dense_matmul():
    X, W, dY = _rand(0, 9, 13), _rand(1, 7, 13), _rand(2, 9, 7)
    ones_o, ones_i = np.ones(7, np.uint8), np.ones(13, np.uint8)
    MW = G.weight_mask_rows(P.row_mask(7, 1, 1), ones_i)
    assert np.array_equal(MW, np.ones((7, 13)))
    assert np.allclose(G.drop_gemm_fwd(X, W, MW, ones_o), np.matmul(X, W.T), rtol=1e-14, atol=1e-14)
    assert np.allclose(G.drop_gemm_bwd_data(dY, W, MW, ones_o), np.matmul(dY, W), rtol=1e-14, atol=1e-14)
    assert np.allclose(G.drop_gemm_bwd_weight(dY, X, MW, ones_o), np.matmul(dY.T, X), rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("dp_o,b_o,dp_i,b_i", [(2, 1, 1, 1), (3, 2, 2, 2), (4, 4, 3, 1), (5, 1, 5, 5)])
def test_row_pattern_equals_compact_product(dp_o, b_o, dp_i, b_i):
    """Section 3.1: the method multiplies the compact matrices and scatters with
    the same pattern; that must equal the masked dense product."""
    B, I, O = 6, 17, 15
    X, W, dY = _rand(3, B, I), _rand(4, O, I), _rand(5, B, O)
    mo, mi = P.row_mask(O, dp_o, b_o), P.row_mask(I, dp_i, b_i)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    alpha = 1.7
    Y = G.drop_gemm_fwd(X, W, MW, mo, alpha)
    Yc = np.zeros_like(Y)
    Yc[:, ko] = alpha * np.matmul(X[:, ki], W[np.ix_(ko, ki)].T)
    assert np.allclose(Y, Yc, rtol=1e-13, atol=1e-13)
    assert np.all(Y[:, mo == 0] == 0.0)                      # dropped outputs exactly zero
    dX = G.drop_gemm_bwd_data(dY, W, MW, mo, alpha)
    dXc = np.zeros_like(dX)
    dXc[:, ki] = alpha * np.matmul(dY[:, ko], W[np.ix_(ko, ki)])
    assert np.allclose(dX, dXc, rtol=1e-13, atol=1e-13)
    assert np.all(dX[:, mi == 0] == 0.0)
    dW = G.drop_gemm_bwd_weight(dY, X, MW, mo, alpha)
    dWc = np.zeros_like(dW)
    dWc[np.ix_(ko, ki)] = alpha * np.matmul(dY[:, ko].T, X[:, ki])
    assert np.allclose(dW, dWc, rtol=1e-13, atol=1e-13)
    assert np.all(dW[MW == 0] == 0.0)
    assert np.allclose(Y, _brute_fwd(X, W, MW, mo, alpha), rtol=1e-13, atol=1e-13)


def test_kept_region_unchanged_by_skipped_work():
    B, I, O = 5, 12, 10
    X, W = _rand(6, B, I), _rand(7, O, I)
    mo = P.row_mask(O, 3, 2)
    Y = G.drop_gemm_fwd(X, W, G.weight_mask_rows(mo, np.ones(I, np.uint8)), mo)
    dense = X @ W.T
    assert np.allclose(Y[:, mo == 1], dense[:, mo == 1], rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("dp,b,x,y", [(2, 1, 4, 4), (3, 2, 4, 2), (4, 1, 2, 8), (7, 5, 4, 4)])
def test_tile_pattern_blockwise(dp, b, x, y):
    """Section 3.2: per output block J only the kept tiles (J,k) contribute."""
    B, I, O = 5, 22, 14
    X, W, dY = _rand(8, B, I), _rand(9, O, I), _rand(10, B, O)
    tm = P.tile_mask(O, I, x, y, dp, b)
    MW = P.expand_tile_mask(tm, O, I, x, y).astype(np.float64)
    ones_o = np.ones(O, np.uint8)
    Y = G.drop_gemm_fwd(X, W, MW, ones_o)
    dX = G.drop_gemm_bwd_data(dY, W, MW, ones_o)
    dW = G.drop_gemm_bwd_weight(dY, X, MW, ones_o)
    Yb, dXb, dWb = np.zeros_like(Y), np.zeros_like(dX), np.zeros_like(dW)
    TR, TC = tm.shape
    for tr in range(TR):
        for tc in range(TC):
            if tm[tr, tc]:
                rs, cs = slice(tr * x, min(O, tr * x + x)), slice(tc * y, min(I, tc * y + y))
                Yb[:, rs] += X[:, cs] @ W[rs, cs].T
                dXb[:, cs] += dY[:, rs] @ W[rs, cs]
                dWb[rs, cs] = dY[:, rs].T @ X[:, cs]
    assert np.allclose(Y, Yb, atol=1e-13) and np.allclose(dX, dXb, atol=1e-13) and np.allclose(dW, dWb, atol=1e-13)
    assert np.all(dW[MW == 0] == 0.0)
    assert np.allclose(Y, _brute_fwd(X, W, MW, ones_o, 1.0), atol=1e-13)


@pytest.mark.parametrize("kind", ["row", "tile"])
def test_backward_is_the_gradient_of_forward(kind):
    """The paper omits the backward formulas; pin them by central differences of
    L = sum(R * Y) with respect to X and W."""
    B, I, O = 4, 9, 8
    X, W, Rm = _rand(11, B, I), _rand(12, O, I), _rand(13, B, O)
    if kind == "row":
        mo, mi = P.row_mask(O, 3, 2), P.row_mask(I, 2, 1)
        MW = G.weight_mask_rows(mo, mi)
    else:
        mo = np.ones(O, np.uint8)
        MW = P.expand_tile_mask(P.tile_mask(O, I, 2, 3, 3, 2), O, I, 2, 3).astype(np.float64)
    alpha = 1.3

    def loss(Xv, Wv):
        return float(np.sum(Rm * G.drop_gemm_fwd(Xv, Wv, MW, mo, alpha)))
    dX = G.drop_gemm_bwd_data(Rm, W, MW, mo, alpha)
    dW = G.drop_gemm_bwd_weight(Rm, X, MW, mo, alpha)
    eps = 1e-6
    for (r, c) in [(0, 0), (1, 3), (3, 8), (2, 5), (0, 1)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[r, c] += eps
        Xm[r, c] -= eps
        assert abs((loss(Xp, W) - loss(Xm, W)) / (2 * eps) - dX[r, c]) < 1e-7
    for (r, c) in [(0, 0), (1, 1), (4, 2), (7, 8), (3, 4), (2, 0), (1, 2)]:
        Wp, Wm_ = W.copy(), W.copy()
        Wp[r, c] += eps
        Wm_[r, c] -= eps
        assert abs((loss(X, Wp) - loss(X, Wm_)) / (2 * eps) - dW[r, c]) < 1e-7


def test_beta_accumulates_old_gradient():
    B, I, O = 3, 6, 5
    X, dY, old = _rand(14, B, I), _rand(15, B, O), _rand(16, O, I)
    mo = P.row_mask(O, 2, 2)
    MW = G.weight_mask_rows(mo, np.ones(I, np.uint8))
    base = G.drop_gemm_bwd_weight(dY, X, MW, mo, 2.0)
    acc = G.drop_gemm_bwd_weight(dY, X, MW, mo, 2.0, beta=0.5, dW_old=old)
    assert np.allclose(acc, base + 0.5 * old, atol=1e-14)


def test_bf16_storage_rounding():
    v = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -3.1415926, 0.0, 1e-30])
    r = R.to_bf16_values(v)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0078125       # ties to even, then up
    assert r[3] == 1.0
    assert abs(r[4] + 3.140625) < 1e-12 and r[5] == 0.0
    # representable in 8 significant bits
    m, _ = np.frexp(r[r != 0])
    assert np.all(m * 256 == np.round(m * 256))


def test_mlp_iteration_against_autograd():
    """The chain (FC -> ReLU, dropout layer skipped) against torch autograd on the
    equivalent masked dense network (library routine as special-case check)."""
    import torch
    rng = np.random.default_rng(17)
    sizes, B = (11, 16, 12, 5), 7
    X0 = rng.uniform(0, 1, (B, sizes[0]))
    Ws = [rng.standard_normal((sizes[l + 1], sizes[l])) * 0.5 for l in range(3)]
    dYL = rng.standard_normal((B, sizes[-1]))
    m_hidden = [P.row_mask(16, 3, 2), P.row_mask(12, 2, 1)]
    out = G.mlp_iteration(X0, Ws, dYL, m_hidden, R.identity)
    tW = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Ws]
    x = torch.tensor(X0, dtype=torch.float64)
    for l in range(3):
        x = x @ tW[l].T
        if l < 2:
            x = torch.relu(x) * torch.tensor(m_hidden[l].astype(np.float64))
    (x * torch.tensor(dYL)).sum().backward()
    assert np.allclose(out["Y"][2], x.detach().numpy(), atol=1e-12)
    for l in range(3):
        assert np.allclose(out["dW"][l], tW[l].grad.numpy(), atol=1e-11), l
    # dropped hidden units: exact zeros in activations, their weight rows/cols get zero gradient
    assert np.all(out["Y"][0][:, m_hidden[0] == 0] == 0)
    assert np.all(out["dW"][1][:, m_hidden[0] == 0] == 0) and np.all(out["dW"][1][m_hidden[1] == 0, :] == 0)


def test_masked_iteration_reduces_to_the_row_pattern_iteration():
    """With MW = outer(m_out, m_in) the synapse-masked chain is the neuron-masked one."""
    rng = np.random.default_rng(23)
    sizes, B = (9, 14, 10, 4), 6
    X0 = rng.uniform(0, 1, (B, sizes[0]))
    Ws = [rng.standard_normal((sizes[l + 1], sizes[l])) * 0.5 for l in range(3)]
    dYL = rng.standard_normal((B, sizes[-1]))
    m = [P.row_mask(14, 3, 1), P.row_mask(10, 2, 2)]
    ones = lambda n: np.ones(n, np.uint8)
    MWs = [G.weight_mask_rows(m[0], ones(9)), G.weight_mask_rows(m[1], m[0]), G.weight_mask_rows(ones(4), m[1])]
    a = G.mlp_iteration(X0, Ws, dYL, m, R.identity)
    b = G.mlp_iteration_masked(X0, Ws, dYL, MWs, R.identity)
    for l in range(3):
        assert np.allclose(a["Y"][l], b["Y"][l], atol=1e-13) and np.allclose(a["dW"][l], b["dW"][l], atol=1e-12)
    for l in range(2):
        assert np.allclose(a["dY"][l], b["dY"][l], atol=1e-12)


def test_masked_iteration_against_autograd():
    """Tile-masked weights on the two hidden layers (Section 3.2) against torch autograd."""
    import torch
    rng = np.random.default_rng(29)
    sizes, B = (12, 16, 8, 5), 5
    X0 = rng.uniform(0, 1, (B, sizes[0]))
    Ws = [rng.standard_normal((sizes[l + 1], sizes[l])) * 0.5 for l in range(3)]
    dYL = rng.standard_normal((B, sizes[-1]))
    MWs = [P.expand_tile_mask(P.tile_mask(16, 12, 4, 4, 3, 2), 16, 12, 4, 4).astype(np.float64),
           P.expand_tile_mask(P.tile_mask(8, 16, 4, 4, 2, 1), 8, 16, 4, 4).astype(np.float64), np.ones((5, 8))]
    out = G.mlp_iteration_masked(X0, Ws, dYL, MWs, R.identity)
    tW = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Ws]
    x = torch.tensor(X0, dtype=torch.float64)
    acts = []
    for l in range(3):
        x = x @ (tW[l] * torch.tensor(MWs[l])).T
        if l < 2:
            x = torch.relu(x)
        x.retain_grad()
        acts.append(x)
    (x * torch.tensor(dYL)).sum().backward()
    assert np.allclose(out["Y"][2], x.detach().numpy(), atol=1e-12)
    for l in range(3):
        assert np.allclose(out["dW"][l], tW[l].grad.numpy(), atol=1e-11), l
        assert np.all(out["dW"][l][MWs[l] == 0] == 0)
    # gradient at a hidden output after the ReLU backward = autograd's gradient at the post-ReLU activation
    # gated by the activation's sign
    for l in range(2):
        assert np.allclose(out["dY"][l], acts[l].grad.numpy() * (acts[l].detach().numpy() > 0), atol=1e-11)
