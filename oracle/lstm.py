"""LSTM layer with a row pattern on its hidden units (test oracle, CPU only, fp64).

Section 7.2.3: the LSTM runs as matrix multiplications, so the same patterns
apply.  Reading (the paper gives no formulas): one 0/1 mask m over the H hidden
units per sequence; the layer is the sub-model LSTM on the kept units.  Fused
weight W[4H x (I+H)], gate blocks of H rows in the order i, f, g, o, columns
[x | h]; no bias; zero initial state.  A dropped unit has zero gate rows, zero
recurrent columns, and h = c = 0 at every step.
"""
import numpy as np


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def masked_weight(W, m, I):
    W = np.asarray(W, dtype=np.float64)
    H = m.shape[0]
    rows = np.tile(m.astype(np.float64), 4)                       # gate rows of each unit
    cols = np.concatenate([np.ones(I), m.astype(np.float64)])     # recurrent columns of each unit
    assert W.shape == (4 * H, I + H)
    return W * np.outer(rows, cols)


def lstm_forward(x, W, m, store):
    """x[T,B,I]; returns dict(h[T,B,H], c[T,B,H], gates[T,B,4H] post-activation).
    `store` rounds h_t where it is stored for the next step's product."""
    x = np.asarray(x, dtype=np.float64)
    T, B, I = x.shape
    H = m.shape[0]
    Wm = masked_weight(W, m, I)
    mf = m.astype(np.float64)[None, :]
    h_prev = np.zeros((B, H))
    c_prev = np.zeros((B, H))
    hs, cs, gs = np.zeros((T, B, H)), np.zeros((T, B, H)), np.zeros((T, B, 4 * H))
    for t in range(T):
        z = np.concatenate([x[t], h_prev], axis=1) @ Wm.T
        i, f = sigmoid(z[:, 0:H]), sigmoid(z[:, H:2 * H])
        g, o = np.tanh(z[:, 2 * H:3 * H]), sigmoid(z[:, 3 * H:4 * H])
        c = mf * (f * c_prev + i * g)
        h = store(mf * (o * np.tanh(c)))
        gs[t] = np.concatenate([i, f, g, o], axis=1)
        hs[t], cs[t] = h, c
        h_prev, c_prev = h, c
    return dict(h=hs, c=cs, gates=gs)


def lstm_backward(x, W, m, fwd, dh_ext, store):
    """Back-propagation through time with the same mask.  dh_ext[T,B,H] is the
    gradient arriving on every h_t.  `store` rounds the gate gradient where it is
    stored as a product operand.  Returns dict(dx[T,B,I], dW[4H, I+H])."""
    x = np.asarray(x, dtype=np.float64)
    T, B, I = x.shape
    H = m.shape[0]
    Wm = masked_weight(W, m, I)
    MW = masked_weight(np.ones_like(Wm), m, I)
    mf = m.astype(np.float64)[None, :]
    hs, cs, gs = fwd["h"], fwd["c"], fwd["gates"]
    dW = np.zeros_like(Wm)
    dx = np.zeros((T, B, I))
    dh_next = np.zeros((B, H))
    dc_next = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        i, f = gs[t][:, 0:H], gs[t][:, H:2 * H]
        g, o = gs[t][:, 2 * H:3 * H], gs[t][:, 3 * H:4 * H]
        c_prev = cs[t - 1] if t > 0 else np.zeros((B, H))
        h_prev = hs[t - 1] if t > 0 else np.zeros((B, H))
        tc = np.tanh(cs[t])
        dh = mf * (np.asarray(dh_ext[t], dtype=np.float64) + dh_next)
        dc = mf * (dc_next + dh * o * (1.0 - tc * tc))
        dgate = store(np.concatenate([
            dc * g * i * (1.0 - i),
            dc * c_prev * f * (1.0 - f),
            dc * i * (1.0 - g * g),
            dh * tc * o * (1.0 - o)], axis=1))
        dc_next = dc * f
        zin = np.concatenate([x[t], h_prev], axis=1)
        dW += (dgate.T @ zin) * MW
        dz = dgate @ Wm
        dx[t] = dz[:, :I]
        dh_next = dz[:, I:]
    return dict(dx=dx, dW=dW)


# ---- tile pattern on the fused weight (Section 3.2 applied to the LSTM of Section 7.2.3) ----
#
# Reading: the "TILE" rows of the LSTM table drop synapses, not units: the tile pattern of Section 3.2 is
# laid over the fused weight W[4H x (I+H)] and every synapse of a dropped tile is absent for the whole
# sequence.  All H units stay alive.  S below is the 0/1 element mask of W (1 = kept).

def lstm_forward_synapse(x, W, S, store):
    """x[T,B,I], W[4H, I+H], S uint8[4H, I+H]; returns dict(h, c, gates) as lstm_forward does."""
    x = np.asarray(x, dtype=np.float64)
    T, B, I = x.shape
    H = W.shape[0] // 4
    assert W.shape == (4 * H, I + H) and S.shape == W.shape
    Ws = np.asarray(W, dtype=np.float64) * S.astype(np.float64)
    h_prev = np.zeros((B, H))
    c_prev = np.zeros((B, H))
    hs, cs, gs = np.zeros((T, B, H)), np.zeros((T, B, H)), np.zeros((T, B, 4 * H))
    for t in range(T):
        z = np.concatenate([x[t], h_prev], axis=1) @ Ws.T
        i, f = sigmoid(z[:, 0:H]), sigmoid(z[:, H:2 * H])
        g, o = np.tanh(z[:, 2 * H:3 * H]), sigmoid(z[:, 3 * H:4 * H])
        c = f * c_prev + i * g
        h = store(o * np.tanh(c))
        gs[t] = np.concatenate([i, f, g, o], axis=1)
        hs[t], cs[t] = h, c
        h_prev, c_prev = h, c
    return dict(h=hs, c=cs, gates=gs)


def lstm_backward_synapse(x, W, S, fwd, dh_ext, store):
    """Back-propagation through time of lstm_forward_synapse; dW is zero on dropped synapses.
    `store` rounds the gate gradient where it is stored as a product operand."""
    x = np.asarray(x, dtype=np.float64)
    T, B, I = x.shape
    H = W.shape[0] // 4
    Sf = S.astype(np.float64)
    Ws = np.asarray(W, dtype=np.float64) * Sf
    hs, cs, gs = fwd["h"], fwd["c"], fwd["gates"]
    dW = np.zeros_like(Ws)
    dx = np.zeros((T, B, I))
    dh_next = np.zeros((B, H))
    dc_next = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        i, f = gs[t][:, 0:H], gs[t][:, H:2 * H]
        g, o = gs[t][:, 2 * H:3 * H], gs[t][:, 3 * H:4 * H]
        c_prev = cs[t - 1] if t > 0 else np.zeros((B, H))
        h_prev = hs[t - 1] if t > 0 else np.zeros((B, H))
        tc = np.tanh(cs[t])
        dh = np.asarray(dh_ext[t], dtype=np.float64) + dh_next
        dc = dc_next + dh * o * (1.0 - tc * tc)
        dgate = store(np.concatenate([
            dc * g * i * (1.0 - i),
            dc * c_prev * f * (1.0 - f),
            dc * i * (1.0 - g * g),
            dh * tc * o * (1.0 - o)], axis=1))
        dc_next = dc * f
        zin = np.concatenate([x[t], h_prev], axis=1)
        dW += (dgate.T @ zin) * Sf
        dz = dgate @ Ws
        dx[t] = dz[:, :I]
        dh_next = dz[:, I:]
    return dict(dx=dx, dW=dW)
