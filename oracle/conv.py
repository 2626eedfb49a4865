"""Convolution with dropped input feature maps (test oracle, CPU only).

Section 5 / Section 6: the CNN variant drops parts of the *input* of a
convolution according to their sensitivity and skips their multiplications;
the binary mask uses 1 = kept.  The workload here takes the channel-level
reading: one sensitivity score per input feature map (mean absolute
activation), the lowest-scoring maps are dropped, and the convolution is the
direct one over the masked input.  NCHW activations, OIHW weights.

Score arithmetic (reading; the paper leaves it open): to make the ranking
independent of summation order the score is an exact integer,
sum over (n,h,w) of floor(min(|a|, 2^15) * 2^24); ranking is by
(score, channel index) ascending, and the first floor(rate*C) are dropped.
"""
import numpy as np

SCORE_SCALE = float(1 << 24)
SCORE_CLAMP = float(1 << 15)


def channel_score_fixed(A) -> np.ndarray:
    """int64[C] exact fixed-point sum of |A| per input channel."""
    A = np.asarray(A, dtype=np.float64)
    q = np.floor(np.minimum(np.abs(A), SCORE_CLAMP) * SCORE_SCALE).astype(np.int64)
    return q.sum(axis=(0, 2, 3))


def channel_mean_abs(A) -> np.ndarray:
    A = np.asarray(A, dtype=np.float64)
    return channel_score_fixed(A) / SCORE_SCALE / (A.shape[0] * A.shape[2] * A.shape[3])


def select_channels(score: np.ndarray, rate: float) -> np.ndarray:
    """uint8[C] mask, 1 = kept: drop the floor(rate*C) channels that come first
    when sorted by (score, index)."""
    C = score.shape[0]
    n_drop = int(np.floor(float(rate) * C))
    order = sorted(range(C), key=lambda c: (int(score[c]), c))
    m = np.ones(C, dtype=np.uint8)
    for c in order[:n_drop]:
        m[c] = 0
    return m


def _out_size(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def conv_fwd(A, Wt, m_c, stride=1, pad=1):
    """Y[n,co,h,w] = sum_{c kept} sum_{kh,kw} A[n,c,h*s+kh-pad,w*s+kw-pad] * Wt[co,c,kh,kw]."""
    A = np.asarray(A, dtype=np.float64) * m_c.astype(np.float64)[None, :, None, None]
    Wt = np.asarray(Wt, dtype=np.float64)
    N, C, H, Wd = A.shape
    Co, _, KH, KW = Wt.shape
    Ho, Wo = _out_size(H, KH, stride, pad), _out_size(Wd, KW, stride, pad)
    Ap = np.zeros((N, C, H + 2 * pad, Wd + 2 * pad))
    Ap[:, :, pad:pad + H, pad:pad + Wd] = A
    Y = np.zeros((N, Co, Ho, Wo))
    for kh in range(KH):
        for kw in range(KW):
            patch = Ap[:, :, kh:kh + (Ho - 1) * stride + 1:stride, kw:kw + (Wo - 1) * stride + 1:stride]
            Y += np.einsum("nchw,oc->nohw", patch, Wt[:, :, kh, kw], optimize=True)
    return Y


def conv_bwd_data(dY, Wt, m_c, in_hw, stride=1, pad=1):
    """dA = (gradient of conv_fwd w.r.t. A) with dropped channels exactly zero."""
    dY = np.asarray(dY, dtype=np.float64)
    Wt = np.asarray(Wt, dtype=np.float64)
    N, Co, Ho, Wo = dY.shape
    _, C, KH, KW = Wt.shape
    H, Wd = in_hw
    dAp = np.zeros((N, C, H + 2 * pad, Wd + 2 * pad))
    for kh in range(KH):
        for kw in range(KW):
            contrib = np.einsum("nohw,oc->nchw", dY, Wt[:, :, kh, kw], optimize=True)
            dAp[:, :, kh:kh + (Ho - 1) * stride + 1:stride, kw:kw + (Wo - 1) * stride + 1:stride] += contrib
    dA = dAp[:, :, pad:pad + H, pad:pad + Wd]
    return dA * m_c.astype(np.float64)[None, :, None, None]


def conv_bwd_weight(dY, A, m_c, ksize=(3, 3), stride=1, pad=1):
    """dWt[co,c,kh,kw] = sum_{n,h,w} dY[n,co,h,w] * A[n,c,h*s+kh-pad,w*s+kw-pad], zero for dropped c."""
    dY = np.asarray(dY, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64) * m_c.astype(np.float64)[None, :, None, None]
    N, Co, Ho, Wo = dY.shape
    _, C, H, Wd = A.shape
    KH, KW = ksize
    Ap = np.zeros((N, C, H + 2 * pad, Wd + 2 * pad))
    Ap[:, :, pad:pad + H, pad:pad + Wd] = A
    dW = np.zeros((Co, C, KH, KW))
    for kh in range(KH):
        for kw in range(KW):
            patch = Ap[:, :, kh:kh + (Ho - 1) * stride + 1:stride, kw:kw + (Wo - 1) * stride + 1:stride]
            dW[:, :, kh, kw] = np.einsum("nohw,nchw->oc", dY, patch, optimize=True)
    return dW * m_c.astype(np.float64)[None, :, None, None]
