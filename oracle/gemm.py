"""Masked dense GEMMs of a fully connected layer under a dropout pattern
(test oracle, CPU only, fp64).

Layout: X[B x I], W[O x I] (a row of W = one output neuron of this layer,
Section 3.1), Y[B x O] = X . W^T.  The pattern is applied as a materialised 0/1
mask on W (Sections 3.1, 3.2, 6): the method only skips multiplications by
zero, so its exact result is the dense product with the masked weight, with the
dropped part of the output set to zero (Section 3.1).  The paper never writes
the backward formulas; they are the ordinary derivatives of this masked layer.

alpha is a caller-chosen scale (e.g. the 1/(1-p) of inverted dropout, which the
paper does not mention); the oracle never picks one.
"""
import numpy as np


def weight_mask_rows(m_out: np.ndarray, m_in: np.ndarray) -> np.ndarray:
    """Row pattern: synapse (o, i) survives iff output neuron o (this layer's
    pattern) and input neuron i (previous layer's pattern) both survive."""
    return np.outer(m_out.astype(np.float64), m_in.astype(np.float64))


def drop_gemm_fwd(X, W, MW, m_out, alpha=1.0, relu=False):
    X = np.asarray(X, dtype=np.float64)
    Wm = np.asarray(W, dtype=np.float64) * MW
    Y = alpha * (X @ Wm.T)
    Y[:, np.asarray(m_out) == 0] = 0.0
    if relu:
        Y = np.maximum(Y, 0.0)
    return Y


def drop_gemm_bwd_data(dY, W, MW, m_out, alpha=1.0):
    dYm = np.asarray(dY, dtype=np.float64) * np.asarray(m_out, dtype=np.float64)[None, :]
    Wm = np.asarray(W, dtype=np.float64) * MW
    return alpha * (dYm @ Wm)


def drop_gemm_bwd_weight(dY, X, MW, m_out, alpha=1.0, beta=0.0, dW_old=None):
    dYm = np.asarray(dY, dtype=np.float64) * np.asarray(m_out, dtype=np.float64)[None, :]
    dW = alpha * (dYm.T @ np.asarray(X, dtype=np.float64)) * MW
    if beta != 0.0:
        dW = dW + beta * np.asarray(dW_old, dtype=np.float64)
    return dW


def relu_bwd(dY, Y):
    """Gradient through ReLU: passes where the stored activation is positive."""
    return np.asarray(dY, dtype=np.float64) * (np.asarray(Y) > 0)


def mlp_iteration(X0, Ws, dYL, m_hidden, store):
    """One training iteration of an MLP with a row pattern on every hidden layer
    (Sections 3.1, 3.2 last paragraph: FC -> activation, dropout layer skipped).

    Ws[l] is W_{l+1}[O x I]; m_hidden[l] is the 0/1 mask of hidden layer l+1's
    neurons (len(Ws)-1 masks; the output layer is not dropped).  `store` is the
    rounding applied where a tensor is stored between two products.
    Returns dict with per-layer inputs X[l], outputs Y[l], dYs[l] (gradient at
    layer l's output after ReLU backward), dXs[l], dWs[l].
    """
    L = len(Ws)
    Xs, Ys = [np.asarray(X0, dtype=np.float64)], []
    masks_in = [np.ones(Ws[0].shape[1], dtype=np.uint8)]
    masks_out = []
    for l in range(L):
        m_out = m_hidden[l] if l < L - 1 else np.ones(Ws[l].shape[0], dtype=np.uint8)
        masks_out.append(m_out)
        MW = weight_mask_rows(m_out, masks_in[l])
        Y = store(drop_gemm_fwd(Xs[l], Ws[l], MW, m_out, relu=(l < L - 1)))
        Ys.append(Y)
        if l < L - 1:
            Xs.append(Y)
            masks_in.append(m_out)
    dYs, dXs, dWs = [None] * L, [None] * L, [None] * L
    dYs[L - 1] = np.asarray(dYL, dtype=np.float64)
    for l in range(L - 1, -1, -1):
        MW = weight_mask_rows(masks_out[l], masks_in[l])
        dWs[l] = store(drop_gemm_bwd_weight(dYs[l], Xs[l], MW, masks_out[l]))
        if l > 0:
            dXs[l] = store(drop_gemm_bwd_data(dYs[l], Ws[l], MW, masks_out[l]))
            dYs[l - 1] = store(relu_bwd(dXs[l], Ys[l - 1]))
    return dict(X=Xs, Y=Ys, dY=dYs, dX=dXs, dW=dWs, m_in=masks_in, m_out=masks_out)


def mlp_iteration_masked(X0, Ws, dYL, MWs, store):
    """The same iteration with an explicit 0/1 mask MWs[l] on every weight matrix
    (tile patterns, Section 3.2: synapses are dropped tile by tile, no neuron is;
    a layer without a pattern gets a mask of ones).  ReLU after every layer but
    the last; `store` as in mlp_iteration.  Returns dict(Y, dY, dW): Y[l] the
    stored output of layer l, dY[l] the gradient at that output (after the ReLU
    backward), dW[l] the weight gradient, zero on dropped synapses.
    """
    L = len(Ws)
    Xs, Ys = [np.asarray(X0, dtype=np.float64)], []
    for l in range(L):
        Wm = np.asarray(Ws[l], dtype=np.float64) * MWs[l]
        Y = Xs[l] @ Wm.T
        if l < L - 1:
            Y = np.maximum(Y, 0.0)
        Y = store(Y)
        Ys.append(Y)
        Xs.append(Y)
    dYs, dWs = [None] * L, [None] * L
    dYs[L - 1] = np.asarray(dYL, dtype=np.float64)
    for l in range(L - 1, -1, -1):
        dWs[l] = store((dYs[l].T @ Xs[l]) * MWs[l])
        if l > 0:
            Wm = np.asarray(Ws[l], dtype=np.float64) * MWs[l]
            dYs[l - 1] = store(relu_bwd(store(dYs[l] @ Wm), Ys[l - 1]))
    return dict(Y=Ys, dY=dYs, dW=dWs)
