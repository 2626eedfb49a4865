"""Pins for the sensitivity prediction and the row- / block-based sensitivity-aware patterns
(Sections 5.1, 5.2.1, 5.2.2, 6)."""
import json
import os

import numpy as np
import pytest

from oracle import conv as OC
from oracle import sampler
from oracle import sensitivity as S


def test_draws_extend_the_pinned_mixer():
    """draw_u32 is the sampler's chain (pinned to published SplitMix64 outputs) with one more link."""
    for seed, it, st, idx in [(0, 0, 1, 0), (5, 17, S.STREAM_ROWS, 123456), (2**63, 2**40, 7, 2**33 + 1)]:
        r1, r2 = sampler.draw_words(seed, it, st)
        h = (r1 << 32) | r2
        assert S.draw_u32(seed, it, st, idx) == sampler.mix64(((h ^ idx) + sampler.GOLDEN) & sampler.M64) >> 32
    u = np.array([S.draw_u32(3, 1, S.STREAM_ROWS, i) for i in range(20000)], dtype=np.float64) / 2.0**32
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / 20000) and abs((u < 0.3).mean() - 0.3) < 4 * np.sqrt(0.21 / 20000)
    assert S.prob_threshold(0.0) == 0 and S.prob_threshold(1.0) == 1 << 32 and S.prob_threshold(0.5) == 1 << 31


def test_input_matrix_is_im2col():
    """Rows = output positions, columns = (c, kh, kw): X @ Wmat^T is the direct convolution (pinned oracle)."""
    rng = np.random.default_rng(3)
    A, Wt = rng.standard_normal((2, 3, 6, 5)), rng.standard_normal((4, 3, 3, 3))
    for stride, pad in ((1, 1), (2, 1), (1, 0)):
        Y = OC.conv_fwd(A, Wt, np.ones(3, np.uint8), stride, pad)
        for n in range(2):
            X = S.input_matrix(A[n], (3, 3), stride, pad)
            assert X.shape == (Y.shape[2] * Y.shape[3], 27)
            assert np.allclose((X @ Wt.reshape(4, -1).T).T.reshape(Y.shape[1:]), Y[n], atol=1e-12)
    # the column order is (c, kh, kw): entry of channel 2, tap (1, 0) at output position (2, 3), pad 1
    X = S.input_matrix(A[0], (3, 3), 1, 1)
    assert X[2 * 5 + 3, (2 * 3 + 1) * 3 + 0] == A[0, 2, 2, 2]


def test_worked_example_of_section_5_1():
    """k = 30 %, threshold 0.5, t = 50 %: a region whose values are mostly above 0.5 is sensitive; all-high and
    all-low regions are decided whatever the sample is; the sample size is floor(k * size)."""
    X = np.full((8, 12), 0.9)
    X[:, 6:] = 0.1
    cnt, smp = S.region_counts(X, 4, 6, 300, 0.5, seed=1, iteration=0, image=0)
    assert smp.tolist() == [[7, 7], [7, 7]]                    # floor(0.3 * 24)
    assert cnt.tolist() == [[7, 0], [7, 0]]
    assert S.sensitive_regions(cnt, smp, 500).tolist() == [[1, 0], [1, 0]]
    # a region with 75 % of its values above the threshold: sensitive at t = 50 % in the vast majority of draws
    rng = np.random.default_rng(0)
    hits = 0
    for it in range(200):
        Xr = np.where(rng.random((10, 10)) < 0.75, 0.8, 0.2)
        c, s = S.region_counts(Xr, 10, 10, 300, 0.5, seed=9, iteration=it, image=0)
        assert s[0, 0] == 30
        hits += int(S.sensitive_regions(c, s, 500)[0, 0])
    assert hits >= 195
    # exactly at the boundary: count * 1000 >= t * s
    assert S.sensitive_regions(np.array([[15]]), np.array([[30]]), 500)[0, 0] == 1
    assert S.sensitive_regions(np.array([[14]]), np.array([[30]]), 500)[0, 0] == 0


def test_sampling_is_uniform_over_the_region_and_clips_edges():
    X = np.zeros((5, 7))
    X[4, 6] = 1.0                                              # only the last element of the clipped region
    tot = 0
    for it in range(4000):
        c, s = S.region_counts(X, 4, 4, 1000, 0.5, seed=4, iteration=it, image=0)
        assert s.tolist() == [[16, 12], [4, 3]]                # sizes of the clipped regions at k = 100 %
        tot += int(c[1, 1])
        assert c[0, 0] == c[0, 1] == c[1, 0] == 0
    # element hit with probability 1/3 per draw, 3 draws per iteration
    assert abs(tot / (4000 * 3) - 1 / 3) < 4 * np.sqrt((1 / 3) * (2 / 3) / 12000)


def test_row_mask_example_of_section_6(golden_dir):
    """Six rows, rows 1, 3, 4 sensitive, 2, 5, 6 insensitive: with m = 0 and n = 1 the mask is the paper's
    1,0,1,1,0,0 (1 = kept); the possibilities are met in frequency otherwise."""
    with open(os.path.join(golden_dir, "paper_examples.json")) as f:
        g = json.load(f)["cnn_row_mask"]
    sens = np.array([1, 0, 1, 1, 0, 0], np.uint8)
    assert S.rsdp_row_mask(sens, 1, 6, 0.0, 1.0, seed=0, iteration=0, image=0).tolist() == g["mask"]
    drops = np.zeros(6)
    T = 6000
    for it in range(T):
        drops += 1 - S.rsdp_row_mask(sens, 1, 6, 0.2, 0.7, seed=11, iteration=it, image=0)
    for p in range(6):
        want = 0.2 if sens[p] else 0.7
        assert abs(drops[p] / T - want) < 4 * np.sqrt(want * (1 - want) / T)
    # bands of x rows share their band's possibility; images draw independently
    k0 = S.rsdp_row_mask(np.array([1, 0], np.uint8), 3, 6, 0.0, 1.0, 0, 0, image=0)
    assert k0.tolist() == [1, 1, 1, 0, 0, 0]
    a = S.rsdp_row_mask(sens, 1, 6, 0.5, 0.5, 3, 4, image=0)
    b = S.rsdp_row_mask(sens, 1, 6, 0.5, 0.5, 3, 4, image=0)
    assert a.tolist() == b.tolist()


def test_balancing_gives_every_group_the_same_number_of_sensitive_blocks():
    rng = np.random.default_rng(5)
    cnt = rng.integers(0, 11, (6, 9))
    smp = np.full((6, 9), 10)
    sens = S.sensitive_regions(cnt, smp, 500)
    bal, Sn = S.balance_groups(cnt, smp, sens)
    assert Sn == int(np.floor(sens.sum() / 6 + 0.5))
    assert np.all(bal.sum(axis=1) == Sn)
    for rb in range(6):                                      # the chosen blocks are the group's highest shares
        chosen, rest = cnt[rb][bal[rb] == 1], cnt[rb][bal[rb] == 0]
        assert chosen.min() >= rest.max()
    # ties: the lower column block wins; unequal sample sizes compare shares, not counts
    b2, _ = S.balance_groups(np.array([[3, 3, 3, 0]]), np.array([[10, 10, 10, 10]]), np.array([[1, 1, 0, 0]], np.uint8))
    assert b2.tolist() == [[1, 1, 0, 0]]
    b3, _ = S.balance_groups(np.array([[3, 2]]), np.array([[10, 4]]), np.array([[1, 0]], np.uint8))
    assert b3.tolist() == [[0, 1]]                           # 2/4 > 3/10
    # already balanced input stays as it is
    even = np.array([[1, 0, 1], [0, 1, 1]], np.uint8)
    assert S.balance_groups(np.array([[9, 1, 8], [2, 9, 7]]), np.full((2, 3), 10), even)[0].tolist() == even.tolist()


def test_block_mask_frequencies():
    sens = np.array([[1, 0, 0], [0, 1, 0]], np.uint8)
    drops = np.zeros((2, 3))
    T = 5000
    for it in range(T):
        drops += 1 - S.bsdp_block_mask(sens, 0.1, 0.6, seed=2, iteration=it, image=1)
    want = np.where(sens == 1, 0.1, 0.6)
    assert np.all(np.abs(drops / T - want) < 4 * np.sqrt(want * (1 - want) / T))


def test_forward_under_row_and_block_masks():
    """RSDP output = the direct convolution with the dropped positions zeroed; BSDP = the matrix product with
    the dropped blocks zeroed, against loops written out."""
    rng = np.random.default_rng(8)
    A, Wt = rng.standard_normal((2, 3, 5, 4)), rng.standard_normal((4, 3, 3, 3))
    full = OC.conv_fwd(A, Wt, np.ones(3, np.uint8), 1, 1)
    keep = (rng.random((2, 20)) < 0.6).astype(np.uint8)
    Y = S.conv_fwd_rows(A, Wt, keep, 1, 1)
    assert np.allclose(Y, full * keep.reshape(2, 1, 5, 4), atol=1e-12)
    assert np.all(Y.reshape(2, 4, 20)[:, :, :][np.broadcast_to((keep == 0)[:, None, :], (2, 4, 20))] == 0)
    x, y = 3, 5
    bk = (rng.random((2, 7, 6)) < 0.5).astype(np.uint8)
    Yb = S.conv_fwd_blocks(A, Wt, bk, x, y, 1, 1)
    Wm = Wt.reshape(4, -1)
    for n in range(2):
        X = S.input_matrix(A[n], (3, 3), 1, 1)
        for co in (0, 3):
            for p in (0, 7, 19):
                ref = sum(X[p, q] * Wm[co, q] for q in range(27) if bk[n, p // x, q // y])
                assert abs(Yb[n, co, p // 4, p % 4] - ref) < 1e-12
    assert np.allclose(S.conv_fwd_blocks(A, Wt, np.ones((2, 7, 6), np.uint8), x, y, 1, 1), full, atol=1e-12)


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (1, 0, 2), (1, 2, 5)])
def test_row_pattern_gradients_are_autograd_of_the_masked_convolution(stride, pad, k):
    """Y = (row kept) * conv(A, W): torch's convolution and autograd on the output masked position by position."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(10 + stride + pad + k)
    N, C, H, W, Co = 2, 3, 7, 6, 4
    A = rng.standard_normal((N, C, H, W))
    Wt = rng.standard_normal((Co, C, k, k))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    keep = (rng.uniform(size=(N, Ho * Wo)) < 0.6).astype(np.uint8)
    keep[0, 0], keep[1, -1] = 1, 0
    dY = rng.standard_normal((N, Co, Ho, Wo))
    At, Wtt = torch.tensor(A, requires_grad=True), torch.tensor(Wt, requires_grad=True)
    Y = F.conv2d(At, Wtt, stride=stride, padding=pad) * torch.tensor(keep.reshape(N, 1, Ho, Wo).astype(np.float64))
    assert np.allclose(S.conv_fwd_rows(A, Wt, keep, stride, pad), Y.detach().numpy(), atol=1e-12)
    (Y * torch.tensor(dY)).sum().backward()
    dA, dW = S.conv_bwd_rows(dY, A, Wt, keep, stride, pad)
    assert np.allclose(dA, At.grad.numpy(), atol=1e-11)
    assert np.allclose(dW, Wtt.grad.numpy(), atol=1e-11)


def test_row_pattern_gradients_special_cases():
    """All rows kept: the plain convolution's gradients (oracle/conv.py).  No row kept: zero.  Gradient arriving
    on a dropped position has no influence."""
    rng = np.random.default_rng(21)
    N, C, H, W, Co = 2, 4, 6, 6, 3
    A, Wt, dY = rng.standard_normal((N, C, H, W)), rng.standard_normal((Co, C, 3, 3)), rng.standard_normal((N, Co, 6, 6))
    ones = np.ones((N, 36), np.uint8)
    dA, dW = S.conv_bwd_rows(dY, A, Wt, ones)
    allc = np.ones(C, np.uint8)
    assert np.allclose(dA, OC.conv_bwd_data(dY, Wt, allc, (H, W)), atol=1e-11)
    assert np.allclose(dW, OC.conv_bwd_weight(dY, A, allc), atol=1e-11)
    dA0, dW0 = S.conv_bwd_rows(dY, A, Wt, np.zeros((N, 36), np.uint8))
    assert not dA0.any() and not dW0.any()
    keep = (rng.uniform(size=(N, 36)) < 0.5).astype(np.uint8)
    dY2 = dY + 9.0 * (1 - keep.reshape(N, 1, 6, 6))
    a1, w1 = S.conv_bwd_rows(dY, A, Wt, keep)
    a2, w2 = S.conv_bwd_rows(dY2, A, Wt, keep)
    assert np.array_equal(a1, a2) and np.array_equal(w1, w2)
    assert not np.allclose(a1, dA)


@pytest.mark.parametrize("stride,pad,k,x,y", [(1, 1, 3, 3, 5), (2, 1, 3, 4, 9), (1, 0, 2, 7, 2), (1, 2, 5, 5, 25)])
def test_block_pattern_gradients_are_autograd_of_the_masked_product(stride, pad, k, x, y):
    """Y_n = W (unfold(A_n) * M): torch's unfold and autograd, with the mask spread entry by entry in loops."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(40 + stride + pad + k)
    N, C, H, W, Co = 2, 3, 7, 6, 4
    A = rng.standard_normal((N, C, H, W))
    Wt = rng.standard_normal((Co, C, k, k))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    R, Q = Ho * Wo, C * k * k
    RB, CB = -(-R // x), -(-Q // y)
    bk = (rng.uniform(size=(N, RB, CB)) < 0.55).astype(np.uint8)
    M = np.zeros((N, Q, R))
    for n in range(N):
        for q in range(Q):
            for p in range(R):
                M[n, q, p] = bk[n, p // x, q // y]
    dY = rng.standard_normal((N, Co, Ho, Wo))
    At, Wtt = torch.tensor(A, requires_grad=True), torch.tensor(Wt, requires_grad=True)
    cols = F.unfold(At, (k, k), padding=pad, stride=stride) * torch.tensor(M)        # [N, C*k*k, Ho*Wo]
    Y = (Wtt.reshape(Co, Q) @ cols).reshape(N, Co, Ho, Wo)
    assert np.allclose(S.conv_fwd_blocks(A, Wt, bk, x, y, stride, pad), Y.detach().numpy(), atol=1e-11)
    (Y * torch.tensor(dY)).sum().backward()
    dA, dW = S.conv_bwd_blocks(dY, A, Wt, bk, x, y, stride, pad)
    assert np.allclose(dA, At.grad.numpy(), atol=1e-11)
    assert np.allclose(dW, Wtt.grad.numpy(), atol=1e-11)


def test_block_pattern_gradients_special_cases():
    """Every block kept: the plain convolution's gradients.  None kept: zero.  Whole block rows dropped: the
    row pattern's gradients.  Blocks of one channel's taps over all rows of an image: that channel dropped in
    that image.  One entry by brute force."""
    rng = np.random.default_rng(22)
    N, C, H, W, Co = 2, 4, 6, 6, 3
    A, Wt, dY = rng.standard_normal((N, C, H, W)), rng.standard_normal((Co, C, 3, 3)), rng.standard_normal((N, Co, 6, 6))
    allc = np.ones(C, np.uint8)
    dA, dW = S.conv_bwd_blocks(dY, A, Wt, np.ones((N, 9, 8), np.uint8), 4, 5)
    assert np.allclose(dA, OC.conv_bwd_data(dY, Wt, allc, (H, W)), atol=1e-11)
    assert np.allclose(dW, OC.conv_bwd_weight(dY, A, allc), atol=1e-11)
    dA0, dW0 = S.conv_bwd_blocks(dY, A, Wt, np.zeros((N, 9, 8), np.uint8), 4, 5)
    assert not dA0.any() and not dW0.any()
    # block rows: bands of 4 rows, kept or dropped as a whole
    band = (rng.uniform(size=(N, 9)) < 0.5).astype(np.uint8)
    a1, w1 = S.conv_bwd_blocks(dY, A, Wt, np.repeat(band[:, :, None], 8, axis=2), 4, 5)
    a2, w2 = S.conv_bwd_rows(dY, A, Wt, np.repeat(band, 4, axis=1))
    assert np.allclose(a1, a2, atol=1e-12) and np.allclose(w1, w2, atol=1e-12)
    # block columns of 9 = one channel's taps, one band of 36 rows = the whole image
    ch = np.array([[1, 0, 1, 1], [0, 1, 1, 0]], np.uint8)
    a3, w3 = S.conv_bwd_blocks(dY, A, Wt, ch[:, None, :], 36, 9)
    for n in range(N):
        an = OC.conv_bwd_data(dY[n:n + 1], Wt, ch[n], (H, W))
        assert np.allclose(a3[n], an[0], atol=1e-11)
        assert not a3[n][ch[n] == 0].any()
    wsum = sum(OC.conv_bwd_weight(dY[n:n + 1], A[n:n + 1], ch[n]) for n in range(N))
    assert np.allclose(w3, wsum, atol=1e-11)
    # brute force: dW[co, c, kh, kw] and dA[n, c, ih, iw] of a random mask
    bk = (rng.uniform(size=(N, 9, 8)) < 0.5).astype(np.uint8)
    a4, w4 = S.conv_bwd_blocks(dY, A, Wt, bk, 4, 5)
    for (co, c, kh, kw) in [(0, 0, 0, 0), (2, 3, 1, 2), (1, 2, 2, 1)]:
        q = (c * 3 + kh) * 3 + kw
        ref = 0.0
        for n in range(N):
            for oh in range(6):
                for ow in range(6):
                    ih, iw = oh + kh - 1, ow + kw - 1
                    if 0 <= ih < 6 and 0 <= iw < 6 and bk[n, (oh * 6 + ow) // 4, q // 5]:
                        ref += dY[n, co, oh, ow] * A[n, c, ih, iw]
        assert abs(w4[co, c, kh, kw] - ref) < 1e-11
    for (n, c, ih, iw) in [(0, 0, 0, 0), (1, 3, 5, 2), (0, 2, 3, 3)]:
        ref = 0.0
        for kh in range(3):
            for kw in range(3):
                oh, ow = ih - kh + 1, iw - kw + 1
                q = (c * 3 + kh) * 3 + kw
                if 0 <= oh < 6 and 0 <= ow < 6 and bk[n, (oh * 6 + ow) // 4, q // 5]:
                    ref += sum(dY[n, co, oh, ow] * Wt[co, c, kh, kw] for co in range(Co))
        assert abs(a4[n, c, ih, iw] - ref) < 1e-11
