"""Region-level sensitivity prediction and the row- / block-based sensitivity-aware dropout
patterns of the CNN variant (Sections 5.1, 5.2.1, 5.2.2; test oracle, CPU only).

The input matrix of one image (Section 5.1, step 1) has one row per output position
p = oh * Wo + ow and one column per (c, kh, kw), q = (c * KH + kh) * KW + kw; its entries are the
zero-padded activations A[c, oh*s + kh - pad, ow*s + kw - pad].  It is cut into x-by-y regions
(edge regions clipped): row band rb = p // x, column block cb = q // y.

Readings taken where the paper leaves the procedure open (each draw is counter-based and integer
only, so that masks can be reproduced bit for bit):
  * the k% sample of a region (step 2): s = max(1, floor(k_permille * size / 1000)) draws WITH
    replacement, draw j picks element e = (u * size) >> 32 of the region in row-major order, u the
    32-bit draw for index (region * 65536 + j) of stream STREAM_SAMPLE.
  * the share t% of the sample that must exceed the threshold (step 3): sensitive iff 1000 * count >= t_permille * s.
  * possibilities m (sensitive) < n (insensitive) become 32-bit thresholds floor(p * 2^32) (p = 1 -> 2^32);
    a unit is DROPPED iff its draw u < threshold.
  * RSDP (Section 5.2.1): the unit is a row of the input matrix; regions span the whole width
    (y = number of columns), so every row band has one sensitivity, shared by its rows.
  * BSDP (Section 5.2.2): the unit is an x-by-y block; the blocks of one row band form a group.
    Balancing: S = the mean number of sensitive blocks per group, rounded half up; in every
    group the S blocks with the largest share of sampled values above the threshold (ties: lower
    column block first) are the sensitive ones, so every group holds the same number.
The 32-bit draw of (seed, iteration, stream, index) chains the SplitMix64 finaliser of oracle/sampler.py
once more over the index.
"""
import numpy as np

from oracle.sampler import GOLDEN, M64, mix64

STREAM_SAMPLE, STREAM_ROWS, STREAM_BLOCKS = 0x5E01, 0x5E02, 0x5E03


def draw_u32(seed: int, iteration: int, stream_id: int, index: int) -> int:
    h = mix64((seed + GOLDEN) & M64)
    h = mix64((h ^ (iteration & M64)) + GOLDEN)
    h = mix64((h ^ (stream_id & 0xFFFFFFFF)) + GOLDEN)
    h = mix64((h ^ (index & M64)) + GOLDEN)
    return h >> 32


def prob_threshold(p: float) -> int:
    """Possibility p in [0, 1] as the 32-bit threshold a draw is compared with."""
    return min(1 << 32, max(0, int(np.floor(float(p) * 4294967296.0))))


def input_matrix(A_img, ksize, stride, pad):
    """[(Ho*Wo) x (C*KH*KW)] input matrix of one image A_img[C, H, W] (Section 5.1, step 1)."""
    A_img = np.asarray(A_img, dtype=np.float64)
    C, H, W = A_img.shape
    KH, KW = ksize
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    Ap = np.zeros((C, H + 2 * pad, W + 2 * pad))
    Ap[:, pad:pad + H, pad:pad + W] = A_img
    X = np.zeros((Ho * Wo, C * KH * KW))
    for oh in range(Ho):
        for ow in range(Wo):
            X[oh * Wo + ow] = Ap[:, oh * stride:oh * stride + KH, ow * stride:ow * stride + KW].reshape(-1)
    return X


def region_counts(X, x, y, k_permille, thr, seed, iteration, image):
    """Per region of one image's input matrix: (sampled values above thr, number of samples)."""
    R, Q = X.shape
    RB, CB = -(-R // x), -(-Q // y)
    cnt = np.zeros((RB, CB), dtype=np.int64)
    smp = np.zeros((RB, CB), dtype=np.int64)
    for rb in range(RB):
        for cb in range(CB):
            r0, q0 = rb * x, cb * y
            h, w = min(x, R - r0), min(y, Q - q0)
            size = h * w
            s = max(1, (k_permille * size) // 1000)
            region = (image * RB + rb) * CB + cb
            c = 0
            for j in range(s):
                u = draw_u32(seed, iteration, STREAM_SAMPLE, region * 65536 + j)
                e = (u * size) >> 32
                c += 1 if X[r0 + e // w, q0 + e % w] > thr else 0
            cnt[rb, cb], smp[rb, cb] = c, s
    return cnt, smp


def sensitive_regions(cnt, smp, t_permille):
    """uint8 map, 1 = sensitive (Section 5.1, step 3)."""
    return (1000 * cnt >= t_permille * smp).astype(np.uint8)


def balance_groups(cnt, smp, sens):
    """BSDP: the same number S of sensitive blocks in every group (row band), chosen by the share of
    sampled values above the threshold (Section 5.2.2)."""
    RB, CB = sens.shape
    total = int(sens.sum())
    S = min(CB, (2 * total + RB) // (2 * RB))          # mean per group, rounded half up
    out = np.zeros_like(sens)
    for rb in range(RB):
        # a before b iff cnt_a / smp_a > cnt_b / smp_b (cross-multiplied, exact), ties: lower index first
        order = list(range(CB))
        for i in range(1, CB):                          # insertion sort on the exact comparison
            j = i
            while j > 0:
                a, b = order[j - 1], order[j]
                if int(cnt[rb, b]) * int(smp[rb, a]) > int(cnt[rb, a]) * int(smp[rb, b]):
                    order[j - 1], order[j] = b, a
                    j -= 1
                else:
                    break
        for cb in order[:S]:
            out[rb, cb] = 1
    return out, S


def rsdp_row_mask(sens_band, x, rows, m, n, seed, iteration, image):
    """uint8[rows], 1 = kept: row p is dropped with possibility m if its band is sensitive, n otherwise
    (Section 5.2.1)."""
    tm, tn = prob_threshold(m), prob_threshold(n)
    keep = np.ones(rows, dtype=np.uint8)
    for p in range(rows):
        u = draw_u32(seed, iteration, STREAM_ROWS, image * rows + p)
        if u < (tm if sens_band[p // x] else tn):
            keep[p] = 0
    return keep


def bsdp_block_mask(sens, m, n, seed, iteration, image):
    """uint8[RB, CB], 1 = kept block (Section 5.2.2)."""
    tm, tn = prob_threshold(m), prob_threshold(n)
    RB, CB = sens.shape
    keep = np.ones((RB, CB), dtype=np.uint8)
    for rb in range(RB):
        for cb in range(CB):
            u = draw_u32(seed, iteration, STREAM_BLOCKS, (image * RB + rb) * CB + cb)
            if u < (tm if sens[rb, cb] else tn):
                keep[rb, cb] = 0
    return keep


def conv_fwd_rows(A, Wt, row_keep, stride=1, pad=1):
    """Y[n, co, p] = (input matrix row p kept) ? sum_q X_n[p, q] * Wmat[co, q] : 0, row_keep[N, Ho*Wo]
    (Section 5.2.1: the kept rows are multiplied, the results fill the same rows of the output)."""
    A = np.asarray(A, dtype=np.float64)
    Wt = np.asarray(Wt, dtype=np.float64)
    N = A.shape[0]
    Co, _, KH, KW = Wt.shape
    Wm = Wt.reshape(Co, -1)
    out = []
    for n in range(N):
        X = input_matrix(A[n], (KH, KW), stride, pad)
        Y = (X * row_keep[n].astype(np.float64)[:, None]) @ Wm.T       # [rows x Co]
        out.append(Y.T)
    Ho = (A.shape[2] + 2 * pad - KH) // stride + 1
    Wo = (A.shape[3] + 2 * pad - KW) // stride + 1
    return np.stack(out).reshape(N, Co, Ho, Wo)


def conv_fwd_blocks(A, Wt, block_keep, x, y, stride=1, pad=1):
    """The same product with the input matrix masked block by block, block_keep[N, RB, CB] (Section 5.2.2)."""
    A = np.asarray(A, dtype=np.float64)
    Wt = np.asarray(Wt, dtype=np.float64)
    N = A.shape[0]
    Co, _, KH, KW = Wt.shape
    Wm = Wt.reshape(Co, -1)
    out = []
    for n in range(N):
        X = input_matrix(A[n], (KH, KW), stride, pad)
        R, Q = X.shape
        M = np.kron(block_keep[n].astype(np.float64), np.ones((x, y)))[:R, :Q]
        out.append(((X * M) @ Wm.T).T)
    Ho = (A.shape[2] + 2 * pad - KH) // stride + 1
    Wo = (A.shape[3] + 2 * pad - KW) // stride + 1
    return np.stack(out).reshape(N, Co, Ho, Wo)


def conv_bwd_rows(dY, A, Wt, row_keep, stride=1, pad=1):
    """Gradients of conv_fwd_rows: the product of Section 5.2.1 only involves the kept rows of the input
    matrix, so only those rows carry gradient.  Per image, with G[p, co] = dY[n, co, p] on kept rows p and 0
    on dropped ones:  dWmat[co, q] += sum_p G[p, co] X_n[p, q],  dX_n[p, q] = sum_co G[p, co] Wmat[co, q],
    and dA collects dX_n back through the positions the input matrix was cut from.
    Returns (dA[N, C, H, W], dWt[Co, C, KH, KW])."""
    A = np.asarray(A, dtype=np.float64)
    Wt = np.asarray(Wt, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    N, C, H, W = A.shape
    Co, _, KH, KW = Wt.shape
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    Wm = Wt.reshape(Co, -1)
    dWm = np.zeros_like(Wm)
    dA = np.zeros_like(A)
    for n in range(N):
        X = input_matrix(A[n], (KH, KW), stride, pad)
        G = dY[n].reshape(Co, Ho * Wo).T * row_keep[n].astype(np.float64)[:, None]      # [rows x Co]
        dWm += G.T @ X
        dX = G @ Wm                                                                      # [rows x C*KH*KW]
        dAp = np.zeros((C, H + 2 * pad, W + 2 * pad))
        for oh in range(Ho):
            for ow in range(Wo):
                dAp[:, oh * stride:oh * stride + KH, ow * stride:ow * stride + KW] += dX[oh * Wo + ow].reshape(C, KH, KW)
        dA[n] = dAp[:, pad:pad + H, pad:pad + W]
    return dA, dWm.reshape(Wt.shape)


def conv_bwd_blocks(dY, A, Wt, block_keep, x, y, stride=1, pad=1):
    """Gradients of conv_fwd_blocks (Section 5.2.2): the product runs over the input matrix with the dropped
    blocks removed, so an entry (p, q) of a dropped block neither contributes to the weight gradient nor
    receives gradient.  Per image, with G[p, co] = dY[n, co, p] and M the block mask spread over entries:
    dWmat[co, q] += sum_p G[p, co] (X_n * M)[p, q],  dX_n = (G Wmat) * M,  and dA collects dX_n back through
    the positions the input matrix was cut from.  Returns (dA[N, C, H, W], dWt[Co, C, KH, KW])."""
    A = np.asarray(A, dtype=np.float64)
    Wt = np.asarray(Wt, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    N, C, H, W = A.shape
    Co, _, KH, KW = Wt.shape
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    Wm = Wt.reshape(Co, -1)
    dWm = np.zeros_like(Wm)
    dA = np.zeros_like(A)
    for n in range(N):
        X = input_matrix(A[n], (KH, KW), stride, pad)
        R, Q = X.shape
        M = np.kron(block_keep[n].astype(np.float64), np.ones((x, y)))[:R, :Q]
        G = dY[n].reshape(Co, Ho * Wo).T                                                 # [rows x Co]
        dWm += G.T @ (X * M)
        dX = (G @ Wm) * M                                                                # [rows x C*KH*KW]
        dAp = np.zeros((C, H + 2 * pad, W + 2 * pad))
        for oh in range(Ho):
            for ow in range(Wo):
                dAp[:, oh * stride:oh * stride + KH, ow * stride:ow * stride + KW] += dX[oh * Wo + ow].reshape(C, KH, KW)
        dA[n] = dAp[:, pad:pad + H, pad:pad + W]
    return dA, dWm.reshape(Wt.shape)
