"""Pins for the oracle's feature-map-dropping convolution (Sections 5, 6)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import conv as C


def _setup(seed, N, Ci, Co, H, W, k=3):
    rng = np.random.default_rng(seed)
    A = np.maximum(rng.standard_normal((N, Ci, H, W)), 0)
    Wt = rng.standard_normal((Co, Ci, k, k))
    return A, Wt


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (1, 0, 1), (1, 2, 5)])
def test_rate_zero_is_library_convolution(stride, pad, k):
    A, Wt = _setup(0, 2, 3, 4, 7, 6, k)
    ones = np.ones(3, np.uint8)
    Y = C.conv_fwd(A, Wt, ones, stride, pad)
    tA = torch.tensor(A, requires_grad=True)
    tW = torch.tensor(Wt, requires_grad=True)
    tY = F.conv2d(tA, tW, stride=stride, padding=pad)
    assert np.allclose(Y, tY.detach().numpy(), atol=1e-12)
    dY = np.random.default_rng(1).standard_normal(Y.shape)
    (tY * torch.tensor(dY)).sum().backward()
    assert np.allclose(C.conv_bwd_data(dY, Wt, ones, (7, 6), stride, pad), tA.grad.numpy(), atol=1e-12)
    assert np.allclose(C.conv_bwd_weight(dY, A, ones, (k, k), stride, pad), tW.grad.numpy(), atol=1e-11)


def test_seven_loop_bruteforce_with_dropped_channels():
    N, Ci, Co, H, W = 2, 4, 3, 5, 5
    A, Wt = _setup(2, N, Ci, Co, H, W)
    m = np.array([1, 0, 1, 0], np.uint8)
    Y = C.conv_fwd(A, Wt, m)
    ref = np.zeros_like(Y)
    for n in range(N):
        for co in range(Co):
            for h in range(H):
                for w in range(W):
                    for c in range(Ci):
                        if not m[c]:
                            continue
                        for kh in range(3):
                            for kw in range(3):
                                y, x = h + kh - 1, w + kw - 1
                                if 0 <= y < H and 0 <= x < W:
                                    ref[n, co, h, w] += A[n, c, y, x] * Wt[co, c, kh, kw]
    assert np.allclose(Y, ref, atol=1e-13)
    dY = np.random.default_rng(3).standard_normal(Y.shape)
    dA = C.conv_bwd_data(dY, Wt, m, (H, W))
    dW = C.conv_bwd_weight(dY, A, m)
    assert np.all(dA[:, m == 0] == 0) and np.all(dW[:, m == 0] == 0)     # dropped maps: exact zeros
    # kept channels: same gradient as the dense convolution restricted to them
    ones = np.ones(Ci, np.uint8)
    assert np.allclose(dA[:, m == 1], C.conv_bwd_data(dY, Wt, ones, (H, W))[:, m == 1], atol=1e-13)
    assert np.allclose(dW[:, m == 1], C.conv_bwd_weight(dY, A, ones)[:, m == 1], atol=1e-13)
    # and it is the gradient of the masked forward
    eps = 1e-6
    for idx in [(0, 0, 0, 0), (1, 2, 4, 4), (0, 2, 2, 3)]:
        Ap, Am = A.copy(), A.copy()
        Ap[idx] += eps
        Am[idx] -= eps
        num = (np.sum(dY * C.conv_fwd(Ap, Wt, m)) - np.sum(dY * C.conv_fwd(Am, Wt, m))) / (2 * eps)
        assert abs(num - dA[idx]) < 1e-7


def test_channel_score_mean_of_relu_gaussian():
    """E|ReLU(z)| = 1/sqrt(2 pi) for z ~ N(0,1)."""
    rng = np.random.default_rng(4)
    A = np.maximum(rng.standard_normal((16, 3, 64, 64)), 0)
    s = C.channel_mean_abs(A)
    assert np.all(np.abs(s - 1 / math.sqrt(2 * math.pi)) < 5 * 0.5838 / math.sqrt(16 * 64 * 64))
    # fixed-point score is an exact integer sum: any order gives the same integer
    perm = rng.permutation(16)
    assert np.array_equal(C.channel_score_fixed(A), C.channel_score_fixed(A[perm][:, :, ::-1, ::-1]))
    assert np.allclose(s, np.abs(A).mean(axis=(0, 2, 3)), rtol=0, atol=2.0**-24)


def test_select_lowest_with_ties():
    score = np.array([5, 1, 3, 1, 9, 3], dtype=np.int64)
    assert C.select_channels(score, 0.5).tolist() == [1, 0, 0, 0, 1, 1]     # drops 1,3 then index 2 before 5
    assert C.select_channels(score, 0.0).tolist() == [1] * 6
    assert C.select_channels(score, 0.34).tolist() == [1, 0, 1, 0, 1, 1]    # floor(2.04) = 2
    assert C.select_channels(np.zeros(4, np.int64), 0.5).tolist() == [0, 0, 1, 1]
    assert int(C.select_channels(np.arange(256), 0.5).sum()) == 128
