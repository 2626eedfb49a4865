"""GPU parity of the sensitivity prediction and the sensitivity-aware patterns (Sections 5.1, 5.2): counts,
flags, masks and lists bit-exact against the oracle; the forward convolution over the kept rows within the
float tolerance, dropped positions exactly +0.0."""
import numpy as np
import pytest
import torch

from oracle import sensitivity as S
from paper_2203_05705_amd import binding as ard
from paper_2203_05705_amd import workloads as WL
from util import assert_parity, from_vals, stored, to_dev

pytestmark = pytest.mark.gpu


def _predict_both(Av, Ad, k, stride, pad, x, y, kpm, tpm, thr, seed, it):
    pred = ard.sens_predict(Ad, (k, k), stride, pad, x, y, kpm, tpm, thr, seed, it)
    torch.cuda.synchronize()
    N = Av.shape[0]
    cnts, smps = [], []
    for n in range(N):
        X = S.input_matrix(Av[n], (k, k), stride, pad)
        c, s = S.region_counts(X, x, y if y else X.shape[1], kpm, thr, seed, it, n)
        cnts.append(c)
        smps.append(s)
    cnt, smp = np.stack(cnts), np.stack(smps)
    assert np.array_equal(pred["samples"].cpu().numpy(), smp)
    assert np.array_equal(pred["count"].cpu().numpy(), cnt)
    sens = np.stack([S.sensitive_regions(cnt[n], smp[n], tpm) for n in range(N)])
    assert np.array_equal(pred["sens"].cpu().numpy(), sens)
    return pred, cnt, smp, sens


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,H,W,k,stride,pad,x,y,kpm,tpm", [
    (2, 3, 6, 5, 3, 1, 1, 4, 6, 300, 500),       # the worked example's k = 30 %, t = 50 %; ragged regions
    (3, 8, 9, 9, 3, 1, 1, 8, 0, 300, 500),       # regions span the width (row-based pattern)
    (2, 4, 8, 8, 5, 2, 2, 3, 16, 1000, 250),     # strided 5x5, every element's worth of draws
    (1, 16, 7, 7, 1, 1, 0, 7, 4, 100, 0),        # 1x1, t = 0: everything sensitive
    # planes that are whole 16-byte pieces: the region's footprint is staged in LDS before the draws
    (2, 8, 8, 8, 3, 1, 1, 4, 0, 300, 500),       # bands that start mid-row and wrap into the next output row
    (2, 6, 8, 12, 3, 1, 1, 5, 18, 500, 400),     # column blocks of two channels: footprint channels start above 0
    (2, 4, 8, 8, 3, 2, 1, 3, 0, 700, 300),       # strided
    (3, 8, 16, 8, 5, 1, 2, 40, 0, 200, 500),     # tall bands, 5x5 filter with two rows of padding
    # enough regions for several bands to share one workgroup's copy of their footprint (3 and 7 per workgroup)
    (8, 16, 28, 28, 3, 1, 1, 4, 0, 300, 500),
    (4, 32, 14, 14, 3, 1, 1, 2, 32, 300, 500),
])
def test_prediction_and_patterns_bit_exact(dtype, N, C, H, W, k, stride, pad, x, y, kpm, tpm):
    print(f"sensitivity case {dtype} N={N} C={C} {H}x{W} k={k} s={stride} p={pad} region {x}x{y} k={kpm} t={tpm}", flush=True)
    rng = np.random.default_rng(N * 100 + C)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Ad = from_vals(Av, dtype)
    for it in (0, 7):
        pred, cnt, smp, sens = _predict_both(Av, Ad, k, stride, pad, x, y, kpm, tpm, 0.5, 11, it)
        rows, RB, CB = ard.sens_regions(Av.shape, (k, k), stride, pad, x, y)
        assert sens.shape == (N, RB, CB)
        # block-based pattern with and without balancing
        for balance in (1, 0):
            bp = ard.sens_block_pattern(pred, balance, 0.2, 0.7, 5, it)
            torch.cuda.synchronize()
            for n in range(N):
                want = S.balance_groups(cnt[n], smp[n], sens[n])[0] if balance else sens[n]
                assert np.array_equal(bp["sens"][n].cpu().numpy(), want)
                assert np.array_equal(bp["keep"][n].cpu().numpy(), S.bsdp_block_mask(want, 0.2, 0.7, 5, it, n))
        # row-based pattern from the first column block's flags (regions spanning the width have only one)
        band = pred["sens"][:, :, :1].contiguous()
        rp = ard.sens_row_pattern(band, rows, x, 0.25, 0.75, 3, it)
        torch.cuda.synchronize()
        mask = np.concatenate([S.rsdp_row_mask(sens[n][:, 0], x, rows, 0.25, 0.75, 3, it, n) for n in range(N)])
        assert np.array_equal(rp["mask"].cpu().numpy(), mask)
        keep = np.flatnonzero(mask).astype(np.int32)
        assert int(rp["count"].item()) == len(keep)
        got = rp["keep"].cpu().numpy()
        assert np.array_equal(got[:len(keep)], keep) and np.all(got[len(keep):] == -1)


def test_row_mask_example_of_section_6_on_the_device():
    sens = torch.tensor([1, 0, 1, 1, 0, 0], dtype=torch.uint8, device="cuda").view(1, 6, 1)
    rp = ard.sens_row_pattern(sens, 6, 1, 0.0, 1.0, 0, 0)
    assert rp["mask"].cpu().tolist() == [1, 0, 1, 1, 0, 0] and rp["keep"].cpu().tolist()[:3] == [0, 2, 3]


def _rows_forward_case(dtype, N, C, Cout, H, W, k, stride, pad, x, m, n_, seed):
    print(f"rows forward {dtype} N={N} C={C} Cout={Cout} {H}x{W} k={k} s={stride} p={pad} x={x}", flush=True)
    rng = np.random.default_rng(seed)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Wv = stored(rng.standard_normal((Cout, C, k, k)) * 0.2, dtype)
    Ad, Wd = from_vals(Av, dtype), from_vals(Wv, dtype)
    pred = ard.sens_predict(Ad, (k, k), stride, pad, x, 0, 300, 500, 0.5, seed, 1)
    rows, RB, CB = ard.sens_regions(Av.shape, (k, k), stride, pad, x, 0)
    rp = ard.sens_row_pattern(pred["sens"], rows, x, m, n_, seed, 1)
    nk = int(rp["count"].item())
    mask = rp["mask"].cpu().numpy().reshape(N, rows)
    Y = ard.conv_fwd_rows(Ad, Wd, rp, nk, stride, pad)
    ref = S.conv_fwd_rows(Av, Wv, mask, stride, pad)
    zero = np.broadcast_to((mask == 0).reshape(N, 1, *ref.shape[2:]), ref.shape)
    assert_parity(Y, ref, dtype, zero, "conv rows Y")
    if stride == 1:
        # gradients of the same pass (the library's data gradient is built for stride 1)
        dYv = stored(rng.standard_normal(ref.shape), dtype)
        dA, dWt = ard.conv_bwd_rows(from_vals(dYv, dtype), Ad, Wd, rp, stride, pad)
        rA, rW = S.conv_bwd_rows(dYv, Av, Wv, mask, stride, pad)
        assert_parity(dA, rA, dtype, None, "conv rows dA")
        assert_parity(dWt, rW, dtype, None, "conv rows dWt")
        if dtype == "bf16" and k - 1 == 2 * pad and nk > 0:
            # one workspace for the layer: the weight gradient takes the grid of A the forward pass left and the
            # masked grid of dY the data gradient left -- same results, bit for bit
            ws = torch.empty(ard.conv_workspace_bytes(ard.BF16, N, C, H, W, Cout, k, k, stride, pad), dtype=torch.uint8, device="cuda")
            ard.conv_fwd_rows(Ad, Wd, rp, nk, stride, pad, ws=ws)
            dA2, dWt2 = ard.conv_bwd_rows(from_vals(dYv, dtype), Ad, Wd, rp, stride, pad, ws=ws,
                                          reuse=ard.CONV_REUSE_A | ard.CONV_REUSE_DY)
            torch.cuda.synchronize()
            assert torch.equal(dA2, dA) and torch.equal(dWt2, dWt), "row-pattern gradients differ with shared grids"
    return nk, N * rows


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,Cout,H,W,k,stride,pad,x", [(2, 8, 16, 7, 7, 3, 1, 1, 4), (3, 12, 20, 9, 6, 3, 1, 1, 5),
                                                           (2, 6, 10, 11, 10, 5, 1, 2, 8), (2, 8, 12, 9, 9, 3, 2, 1, 3),
                                                           (5, 24, 130, 10, 12, 3, 1, 1, 16)])
def test_forward_over_the_kept_rows(dtype, N, C, Cout, H, W, k, stride, pad, x):
    _rows_forward_case(dtype, N, C, Cout, H, W, k, stride, pad, x, 0.2, 0.7, seed=N * 10 + C)


def test_forward_over_the_kept_rows_degenerate():
    """Nothing dropped (m = n = 0) equals the plain forward pass; everything dropped gives zeros."""
    nk, tot = _rows_forward_case("bf16", 2, 8, 16, 7, 7, 3, 1, 1, 4, 0.0, 0.0, seed=1)
    assert nk == tot
    nk, _ = _rows_forward_case("bf16", 2, 8, 16, 7, 7, 3, 1, 1, 4, 1.0, 1.0, seed=2)
    assert nk == 0


@pytest.mark.parametrize("m,n_", [(0.05, 0.2), (0.6, 0.9), (1.0, 1.0)])
def test_forward_over_the_kept_rows_both_ways_of_zeroing(m, n_):
    """Planes of whole 16-byte pieces: with most rows kept the dropped positions are zeroed by masked stores, with
    few kept the whole output is zeroed as one stream before the product writes the kept rows; nothing kept: zeros."""
    nk, tot = _rows_forward_case("bf16", 5, 24, 130, 10, 12, 3, 1, 1, 8, m, n_, seed=int(m * 100) + 7)
    if m == 1.0:
        assert nk == 0
    elif m < 0.1:
        assert nk * 10 > tot * 7, (nk, tot)       # the masked stores
    else:
        assert 0 < nk and nk * 10 <= tot * 7, (nk, tot)   # the stream


def test_config5_layer_under_the_row_pattern():
    """The config-5 layer (N=128, C=Cout=256, 28x28, 3x3) under the row-based sensitivity-aware pattern: bands
    of 8 output positions, k = 30 %, threshold 0.5, t = 50 %, possibilities 0.3 / 0.7."""
    wl = WL.conv_layer(seed=5)
    Av, Wv = wl.values("A"), wl.values("Wt")
    Ad, Wd = (to_dev(wl.arrays[k], "bf16") for k in ("A", "Wt"))
    x = 8
    pred = ard.sens_predict(Ad, (3, 3), 1, 1, x, 0, 300, 500, 0.5, 5, 0)
    rows, RB, CB = ard.sens_regions(Av.shape, (3, 3), 1, 1, x, 0)
    # prediction checked on a sample of images (the oracle walks the draws one by one)
    got_c, got_s = pred["count"].cpu().numpy(), pred["sens"].cpu().numpy()
    for n in (0, 57, 127):
        X = S.input_matrix(Av[n], (3, 3), 1, 1)
        Q = X.shape[1]
        for rb in (0, 40, RB - 1):
            r0 = rb * x
            size = min(x, rows - r0) * Q
            sn = max(1, 300 * size // 1000)
            cc = 0
            for j in range(sn):
                e = (S.draw_u32(5, 0, S.STREAM_SAMPLE, ((n * RB + rb) * CB) * 65536 + j) * size) >> 32
                cc += 1 if X[r0 + e // Q, e % Q] > 0.5 else 0
            assert got_c[n, rb, 0] == cc and got_s[n, rb, 0] == (1 if 1000 * cc >= 500 * sn else 0)
    rp = ard.sens_row_pattern(pred["sens"], rows, x, 0.3, 0.7, 5, 0)
    nk = int(rp["count"].item())
    mask = rp["mask"].cpu().numpy().reshape(128, rows)
    want = np.stack([S.rsdp_row_mask(got_s[n][:, 0], x, rows, 0.3, 0.7, 5, 0, n) for n in range(128)])
    assert np.array_equal(mask, want) and nk == int(want.sum())
    print(f"config 5 under the row pattern: {nk} of {128 * rows} positions kept", flush=True)
    Y = ard.conv_fwd_rows(Ad, Wd, rp, nk)
    from oracle import conv as OC
    ref = OC.conv_fwd(Av, Wv, np.ones(256, np.uint8)) * mask.reshape(128, 1, 28, 28)
    zero = np.broadcast_to((mask == 0).reshape(128, 1, 28, 28), ref.shape)
    assert_parity(Y, ref, "bf16", zero, "config 5 rows Y")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,Cout,H,W,k,stride,pad,x,y", [(2, 8, 16, 7, 7, 3, 1, 1, 4, 8), (3, 12, 20, 9, 6, 3, 1, 1, 5, 16),
                                                             (2, 6, 10, 11, 10, 5, 1, 2, 8, 32), (2, 8, 12, 9, 9, 3, 2, 1, 3, 9),
                                                             (4, 24, 130, 10, 12, 3, 1, 1, 16, 64),
                                                             # blocks of whole 64-channel groups over all taps, bands of
                                                             # half a tile or more: dropped blocks are skipped (bf16)
                                                             (2, 128, 200, 12, 12, 3, 1, 1, 72, 576), (3, 100, 140, 12, 13, 3, 1, 1, 78, 576), (3, 100, 100, 12, 13, 3, 1, 1, 156, 576),
                                                             (2, 192, 130, 9, 16, 3, 1, 1, 144, 576), (5, 256, 300, 14, 14, 3, 1, 1, 98, 1152),
                                                             (2, 128, 136, 16, 16, 1, 1, 0, 128, 64), (2, 64, 256, 15, 15, 5, 1, 2, 75, 1600)])
def test_forward_under_the_block_pattern(dtype, N, C, Cout, H, W, k, stride, pad, x, y):
    """Section 5.2.2: prediction per x-by-y region, balanced groups, block mask, forward product over the kept blocks."""
    print(f"blocks forward {dtype} N={N} C={C} Cout={Cout} {H}x{W} k={k} s={stride} p={pad} x={x} y={y}", flush=True)
    rng = np.random.default_rng(N * 7 + C + y)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Wv = stored(rng.standard_normal((Cout, C, k, k)) * 0.2, dtype)
    Ad, Wd = from_vals(Av, dtype), from_vals(Wv, dtype)
    pred = ard.sens_predict(Ad, (k, k), stride, pad, x, y, 300, 500, 0.5, 3, 2)
    rows, RB, CB = ard.sens_regions(Av.shape, (k, k), stride, pad, x, y)
    bp = ard.sens_block_pattern(pred, 1, 0.2, 0.7, 3, 2)
    keep = bp["keep"].cpu().numpy().reshape(N, RB, CB)
    assert 0 < keep.sum() < keep.size
    Y = ard.conv_fwd_blocks(Ad, Wd, bp["keep"], x, y, stride, pad)
    assert_parity(Y, S.conv_fwd_blocks(Av, Wv, keep, x, y, stride, pad), dtype, None, "conv blocks Y")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,Cout,H,W,k,stride,pad,x,y", [(2, 8, 16, 7, 7, 3, 1, 1, 4, 8), (3, 12, 20, 9, 6, 3, 1, 1, 5, 16),
                                                             (2, 6, 10, 11, 10, 5, 1, 2, 8, 32), (2, 8, 12, 9, 9, 3, 2, 1, 3, 9),
                                                             (4, 24, 130, 10, 12, 3, 1, 1, 16, 64), (3, 140, 20, 12, 13, 3, 1, 0, 8, 0),
                                                             (2, 5, 7, 6, 6, 2, 1, 1, 7, 3),
                                                             # blocks of whole channels: one ordinary pass per column block
                                                             (2, 8, 16, 7, 7, 3, 1, 1, 4, 18), (2, 40, 24, 9, 9, 3, 1, 1, 5, 90),
                                                             (2, 37, 12, 8, 8, 3, 1, 1, 6, 90), (3, 128, 136, 12, 12, 3, 1, 1, 72, 576),
                                                             (2, 20, 16, 9, 9, 3, 2, 1, 5, 45)])
def test_gradients_under_the_block_pattern(dtype, N, C, Cout, H, W, k, stride, pad, x, y):
    """Section 5.2.2: gradients of the product over the kept blocks (the data gradient for stride 1 only)."""
    print(f"blocks gradients {dtype} N={N} C={C} Cout={Cout} {H}x{W} k={k} s={stride} p={pad} x={x} y={y}", flush=True)
    rng = np.random.default_rng(N * 11 + C + y)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Wv = stored(rng.standard_normal((Cout, C, k, k)) * 0.2, dtype)
    rows, RB, CB = ard.sens_regions(Av.shape, (k, k), stride, pad, x, y)
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    dYv = stored(rng.standard_normal((N, Cout, Ho, Wo)), dtype)
    keep = (rng.uniform(size=(N, RB, CB)) < 0.5).astype(np.uint8)
    keep[0, 0, 0], keep[-1, -1, -1] = 1, 0
    Ad, Wd, dYd = from_vals(Av, dtype), from_vals(Wv, dtype), from_vals(dYv, dtype)
    kd = torch.from_numpy(keep.reshape(-1)).cuda()
    yy = y if y else C * k * k
    ref_dA, ref_dW = S.conv_bwd_blocks(dYv, Av, Wv, keep, x, yy, stride, pad)
    if stride == 1:
        dA, dW = ard.conv_bwd_blocks(dYd, Ad, Wd, kd, x, y, stride, pad)
        assert_parity(dA, ref_dA, dtype, None, "conv blocks dA")
    else:
        dW = torch.empty_like(Wd)
        ws = torch.empty(ard.conv_workspace_bytes(ard._dtype_code(Ad), N, C, H, W, Cout, k, k, stride, pad), dtype=torch.uint8, device="cuda")
        args = [ard._dtype_code(Ad), N, C, H, W, Cout, k, k, stride, pad, x, y, Ad.data_ptr(), Wd.data_ptr(), dYd.data_ptr(),
                kd.data_ptr()]
        tail = [ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream]
        assert ard.lib().ard_conv_bwd_blocks(ard.CONV_BWD_WEIGHT, *args, dW.data_ptr(), *tail) == 0
        dA = torch.empty_like(Ad)
        assert ard.lib().ard_conv_bwd_blocks(ard.CONV_BWD_DATA, *args, dA.data_ptr(), *tail) == -6  # ARD_EUNSUPPORTED
    torch.cuda.synchronize()
    assert_parity(dW, ref_dW, dtype, None, "conv blocks dW")


@pytest.mark.parametrize("seed", range(8))
def test_block_pattern_random_shapes(seed):
    """Seeded random layers under random block masks: forward and both gradients against the oracle, whichever
    path (skipping, per-column-block passes, general engine) the shape takes."""
    import random
    rnd = random.Random(900 + seed)
    k = rnd.choice((1, 3, 3, 5))
    pad = rnd.choice((0, k // 2))
    H, W = rnd.randint(k + 3, 16), rnd.randint(k + 3, 16)
    N, C, Cout = rnd.randint(1, 3), rnd.choice((8, 40, 64, 100, 128)), rnd.choice((24, 65, 130, 200))
    Ho, Wo = H + 2 * pad - k + 1, W + 2 * pad - k + 1
    x = rnd.choice((rnd.randint(1, Ho * Wo), max(1, Ho * Wo // rnd.randint(1, 3))))
    y = rnd.choice((0, 64 * k * k, k * k * rnd.randint(1, 40), rnd.randint(1, C * k * k)))
    print(f"random blocks case N={N} C={C} Cout={Cout} {H}x{W} k={k} p={pad} x={x} y={y}", flush=True)
    rng = np.random.default_rng(seed)
    dtype = "bf16"
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Wv = stored(rng.standard_normal((Cout, C, k, k)) * 0.2, dtype)
    dYv = stored(rng.standard_normal((N, Cout, Ho, Wo)), dtype)
    rows, RB, CB = ard.sens_regions(Av.shape, (k, k), 1, pad, x, y)
    keep = (rng.uniform(size=(N, RB, CB)) < 0.5).astype(np.uint8)
    Ad, Wd, dYd = from_vals(Av, dtype), from_vals(Wv, dtype), from_vals(dYv, dtype)
    kd = torch.from_numpy(keep.reshape(-1)).cuda()
    yy = y if y else C * k * k
    Y = ard.conv_fwd_blocks(Ad, Wd, kd, x, y, 1, pad)
    dA, dW = ard.conv_bwd_blocks(dYd, Ad, Wd, kd, x, y, 1, pad)
    torch.cuda.synchronize()
    assert_parity(Y, S.conv_fwd_blocks(Av, Wv, keep, x, yy, 1, pad), dtype, None, "random blocks Y")
    ref_dA, ref_dW = S.conv_bwd_blocks(dYv, Av, Wv, keep, x, yy, 1, pad)
    assert_parity(dA, ref_dA, dtype, None, "random blocks dA")
    assert_parity(dW, ref_dW, dtype, None, "random blocks dW")
    # a second call gives the same bits (the order the tiles are placed in may differ between calls, results may not)
    Y2 = ard.conv_fwd_blocks(Ad, Wd, kd, x, y, 1, pad)
    dA2, dW2 = ard.conv_bwd_blocks(dYd, Ad, Wd, kd, x, y, 1, pad)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y) and torch.equal(dA2, dA) and torch.equal(dW2, dW)


def test_forward_under_the_block_pattern_many_tiles():
    """More pixel tiles than the plan ranks (over 2048: they stay in band order): 1100 images of two bands each,
    checked against the oracle on sampled images (first, middle, last)."""
    N, C, Cout, H, W, x, y = 1100, 128, 72, 12, 12, 72, 576
    rng = np.random.default_rng(77)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), "bf16")
    Wv = stored(rng.standard_normal((Cout, C, 3, 3)) * 0.2, "bf16")
    Ad, Wd = from_vals(Av, "bf16"), from_vals(Wv, "bf16")
    pred = ard.sens_predict(Ad, (3, 3), 1, 1, x, y, 300, 500, 0.5, 3, 2)
    rows, RB, CB = ard.sens_regions(Av.shape, (3, 3), 1, 1, x, y)
    assert N * RB > 2048
    bp = ard.sens_block_pattern(pred, 1, 0.3, 0.7, 3, 2)
    keep = bp["keep"].cpu().numpy().reshape(N, RB, CB)
    assert 0.2 < keep.mean() < 0.8
    Y = ard.conv_fwd_blocks(Ad, Wd, bp["keep"], x, y)
    torch.cuda.synchronize()
    idx = [0, 1, 2, 548, 549, 550, 551, 1097, 1098, 1099]
    ref = S.conv_fwd_blocks(Av[idx], Wv, keep[idx], x, y)
    assert_parity(Y[idx], ref, "bf16", None, "conv blocks Y, sampled images")


def test_config5_layer_under_the_block_pattern():
    """The config-5 layer under the block-based pattern: 112-by-576 blocks of the 784 x 2304 input matrices (four
    rows of output positions by one 64-channel group over all taps: the forward pass skips the dropped blocks),
    balanced groups, possibilities 0.3 / 0.7; forward pass and both gradients against the oracle on every element."""
    wl = WL.conv_layer(seed=5)
    Av, Wv, dYv = wl.values("A"), wl.values("Wt"), wl.values("dY")
    Ad, Wd, dYd = (to_dev(wl.arrays[k], "bf16") for k in ("A", "Wt", "dY"))
    x, y = 112, 576
    pred = ard.sens_predict(Ad, (3, 3), 1, 1, x, y, 300, 500, 0.5, 5, 0)
    rows, RB, CB = ard.sens_regions(Av.shape, (3, 3), 1, 1, x, y)
    bp = ard.sens_block_pattern(pred, 1, 0.3, 0.7, 5, 0)
    keep = bp["keep"].cpu().numpy().reshape(128, RB, CB)
    print(f"config 5 under the block pattern: {int(keep.sum())} of {keep.size} blocks kept; running oracle ...", flush=True)
    assert 0.2 < keep.mean() < 0.8
    Y = ard.conv_fwd_blocks(Ad, Wd, bp["keep"], x, y)
    dA, dW = ard.conv_bwd_blocks(dYd, Ad, Wd, bp["keep"], x, y)
    torch.cuda.synchronize()
    Y2 = ard.conv_fwd_blocks(Ad, Wd, bp["keep"], x, y)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y), "two forward calls under the same block mask differ"
    assert_parity(Y, S.conv_fwd_blocks(Av, Wv, keep, x, y), "bf16", None, "config 5 blocks Y")
    ref_dA, ref_dW = S.conv_bwd_blocks(dYv, Av, Wv, keep, x, y)
    assert_parity(dA, ref_dA, "bf16", None, "config 5 blocks dA")
    assert_parity(dW, ref_dW, "bf16", None, "config 5 blocks dW")


@pytest.mark.parametrize("N,rows,x", [(3, 50, 4), (40, 784, 8), (128, 784, 8)])
def test_row_pattern_without_a_mask_and_with_an_unaligned_one(N, rows, x):
    """The kept list and the count do not depend on whether (or where) the mask is written: with a mask the
    list offsets come from its ones, without one (or with one that is not 16-byte aligned) from recounting."""
    rng = np.random.default_rng(N + rows)
    RB = -(-rows // x)
    sens = torch.from_numpy((rng.uniform(size=(N, RB, 1)) < 0.4).astype(np.uint8)).cuda()
    ref = ard.sens_row_pattern(sens, rows, x, 0.25, 0.75, 11, 3)
    nk = int(ref["count"].item())
    lib = ard.lib()
    total = N * rows
    st = torch.cuda.current_stream().cuda_stream
    for variant in ("no mask", "unaligned mask"):
        keep = torch.full((total,), -1, dtype=torch.int32, device="cuda")
        count = torch.zeros(1, dtype=torch.int32, device="cuda")
        buf = torch.zeros(total + 16, dtype=torch.uint8, device="cuda")
        mask_ptr = None if variant == "no mask" else buf.data_ptr() + 3
        rc = lib.ard_sens_row_pattern(N, rows, x, sens.data_ptr(), 0.25, 0.75, 11, 3, mask_ptr, keep.data_ptr(), count.data_ptr(), st)
        torch.cuda.synchronize()
        assert rc == 0 and int(count.item()) == nk, variant
        assert torch.equal(keep, ref["keep"]), variant
        if mask_ptr is not None:
            assert torch.equal(buf[3:3 + total], ref["mask"]) and not buf[:3].any() and not buf[3 + total:].any()
    # the list is the ascending set of ones of the mask
    m = ref["mask"].cpu().numpy()
    assert np.array_equal(ref["keep"].cpu().numpy()[:nk], np.flatnonzero(m)) and nk == int(m.sum())
