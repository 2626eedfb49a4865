"""GPU parity: drop_gemm_fwd / bwd_data / bwd_weight against the masked-dense oracle."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from paper_2203_05705_amd import binding as ard
from paper_2203_05705_amd import workloads as WL
from util import assert_parity, from_vals, stored, to_dev

pytestmark = pytest.mark.gpu


def _masks_row(O, I, po, pi):
    mo = P.row_mask(O, *po) if po else np.ones(O, np.uint8)
    mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
    return mo, mi


def _run_row_case(dtype, B, I, O, po, pi, alpha=1.0, relu=False, beta=0.0, seed=0, use_relu_src=False):
    print(f"row case dtype={dtype} B={B} I={I} O={O} pat_out={po} pat_in={pi} alpha={alpha} relu={relu} beta={beta}",
          flush=True)
    rng = np.random.default_rng(seed)
    Xv, Wv = stored(rng.standard_normal((B, I)), dtype), stored(rng.standard_normal((O, I)) * 0.1, dtype)
    dYv = stored(rng.standard_normal((B, O)), dtype)
    mo, mi = _masks_row(O, I, po, pi)
    MW = G.weight_mask_rows(mo, mi)
    X, W, dY = from_vals(Xv, dtype), from_vals(Wv, dtype), from_vals(dYv, dtype)
    pat_o = ard.Pattern.row(*po) if po else None
    pat_i = ard.Pattern.row(*pi) if pi else None
    torch_dt = X.dtype
    # outputs start poisoned: every element must be written
    Y = torch.full((B, O), float("nan"), dtype=torch_dt, device="cuda")
    ard.drop_gemm_fwd(X, W, pat_o, pat_i, alpha=alpha, relu=relu, out=Y)
    assert_parity(Y, G.drop_gemm_fwd(Xv, Wv, MW, mo, alpha, relu), dtype, zero_mask=(mo == 0)[None, :], what="Y")
    dX = torch.full((B, I), float("nan"), dtype=torch_dt, device="cuda")
    relu_src = None
    ref_dX = G.drop_gemm_bwd_data(dYv, Wv, MW, mo, alpha)
    if use_relu_src:
        src = stored(rng.standard_normal((B, I)), dtype)
        relu_src = from_vals(src, dtype)
        ref_dX = G.relu_bwd(ref_dX, src)
    ard.drop_gemm_bwd_data(dY, W, pat_o, pat_i, alpha=alpha, relu_src=relu_src, out=dX)
    assert_parity(dX, ref_dX, dtype, zero_mask=(mi == 0)[None, :], what="dX")
    if beta != 0.0:
        oldv = stored(rng.standard_normal((O, I)), dtype)
        dW = from_vals(oldv, dtype)
        ref = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo, alpha, beta, oldv)
        ard.drop_gemm_bwd_weight(dY, X, pat_o, pat_i, alpha=alpha, beta=beta, out=dW)
        assert_parity(dW, ref, dtype, what="dW")
    else:
        dW = torch.full((O, I), float("nan"), dtype=torch_dt, device="cuda")
        ard.drop_gemm_bwd_weight(dY, X, pat_o, pat_i, alpha=alpha, out=dW)
        assert_parity(dW, G.drop_gemm_bwd_weight(dYv, Xv, MW, mo, alpha), dtype, zero_mask=(MW == 0), what="dW")
    torch.cuda.synchronize()


def test_config1_mlp_layer_f32():
    """BASELINE config 1: X 64x784, W 1024x784 fp32, row pattern dp=2, offset 0 (b=1), seed 0."""
    wl = WL.mlp_layer_f32(seed=0)
    X, W, dY = (wl.arrays[k] for k in ("X", "W", "dY"))
    B, I, O = wl.params["B"], wl.params["I"], wl.params["O"]
    mo = P.row_mask(O, 2, 1)
    MW = G.weight_mask_rows(mo, np.ones(I, np.uint8))
    pat = ard.Pattern.row(2, 1)
    dX_, dW_ = (torch.full(s, float("nan"), device="cuda") for s in ((B, I), (O, I)))
    Y = ard.drop_gemm_fwd(to_dev(X, "f32"), to_dev(W, "f32"), pat)
    ard.drop_gemm_bwd_data(to_dev(dY, "f32"), to_dev(W, "f32"), pat, out=dX_)
    ard.drop_gemm_bwd_weight(to_dev(dY, "f32"), to_dev(X, "f32"), pat, out=dW_)
    e1 = assert_parity(Y, G.drop_gemm_fwd(X, W, MW, mo), "f32", zero_mask=(mo == 0)[None, :], what="Y")
    e2 = assert_parity(dX_, G.drop_gemm_bwd_data(dY, W, MW, mo), "f32", what="dX")
    e3 = assert_parity(dW_, G.drop_gemm_bwd_weight(dY, X, MW, mo), "f32", zero_mask=(MW == 0), what="dW")
    print(f"config1 max rel err: Y {e1:.2e} dX {e2:.2e} dW {e3:.2e}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,I,O,po,pi", [
    (64, 96, 128, None, None),            # rate 0 == dense
    (37, 100, 83, (2, 1), None),          # ragged everything
    (37, 100, 83, (3, 3), (2, 2)),        # both patterns, b = dp
    (130, 264, 200, (4, 2), (3, 1)),      # several tiles and a tail
    (5, 17, 9, (9, 9), (17, 17)),         # dp = number of units: a single kept row / column
    (200, 784, 300, (5, 4), None),
    (129, 1000, 257, None, (7, 7)),
])
def test_row_pattern_parity(dtype, B, I, O, po, pi):
    _run_row_case(dtype, B, I, O, po, pi, seed=B + I)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_pattern_epilogue_options(dtype):
    _run_row_case(dtype, 70, 136, 90, (2, 2), (2, 1), alpha=2.0, relu=True, beta=0.5, seed=5)
    _run_row_case(dtype, 70, 136, 90, (3, 1), None, alpha=3.0, relu=False, beta=1.0, seed=6, use_relu_src=True)


@pytest.mark.parametrize("B", [700, 61, 1027])
def test_weight_gradient_contracts_a_batch_that_is_no_multiple_of_8(B):
    """16-byte aligned widths, ragged batch: the weight gradient contracts over rows, so its last step
    ends at any row (the forward and data gradient contract along the rows' 16-byte pieces)."""
    _run_row_case("bf16", B, 512, 768, None, None, seed=B)
    _run_row_case("bf16", B, 1024, 640, (2, 2), (3, 1), seed=B + 1)


def test_row_pattern_multi_tile_bf16():
    """Large enough for the 128x128 workgroup tile, ragged in every dimension."""
    _run_row_case("bf16", 1000, 1048, 2050, (2, 1), (2, 2), seed=9)
    _run_row_case("bf16", 1024, 784, 2048, (3, 2), None, relu=True, seed=10)


def test_list_pattern_parity():
    dtype, B, I, O = "bf16", 96, 160, 144
    rng = np.random.default_rng(21)
    mo = (rng.uniform(size=O) < 0.4).astype(np.uint8)
    mi = (rng.uniform(size=I) < 0.6).astype(np.uint8)
    mo[0], mi[-1] = 1, 1
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    X, W, dY = from_vals(Xv, dtype), from_vals(Wv, dtype), from_vals(dYv, dtype)
    po = ard.Pattern.list(torch.from_numpy(P.keep_list(mo)).cuda())
    pi = ard.Pattern.list(torch.from_numpy(P.keep_list(mi)).cuda())
    MW = G.weight_mask_rows(mo, mi)
    assert_parity(ard.drop_gemm_fwd(X, W, po, pi), G.drop_gemm_fwd(Xv, Wv, MW, mo), dtype, (mo == 0)[None, :], "Y")
    assert_parity(ard.drop_gemm_bwd_data(dY, W, po, pi), G.drop_gemm_bwd_data(dYv, Wv, MW, mo), dtype,
                  (mi == 0)[None, :], "dX")
    assert_parity(ard.drop_gemm_bwd_weight(dY, X, po, pi), G.drop_gemm_bwd_weight(dYv, Xv, MW, mo), dtype, MW == 0, "dW")
    # an empty list keeps nothing: outputs are all zero
    empty = ard.Pattern.list(torch.zeros(1, dtype=torch.int32, device="cuda"), count=0)
    Y = torch.full((B, O), float("nan"), dtype=X.dtype, device="cuda")
    ard.drop_gemm_fwd(X, W, empty, None, out=Y)
    assert torch.count_nonzero(Y.view(torch.int16)).item() == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,I,O,x,y,dp,b", [
    (64, 128, 128, 64, 64, 2, 1),
    (100, 256, 192, 64, 64, 3, 2),
    (70, 200, 150, 64, 64, 4, 3),          # clipped edge tiles
    (130, 256, 256, 32, 32, 3, 1),         # the paper's 32x32 tiles
    (64, 320, 256, 128, 64, 5, 5),
    (90, 256, 256, 64, 64, 16, 7),         # some tile rows keep nothing
    (50, 96, 160, 32, 96, 2, 2),
])
def test_tile_pattern_parity(dtype, B, I, O, x, y, dp, b):
    print(f"tile case dtype={dtype} B={B} I={I} O={O} tile={x}x{y} dp={dp} b={b}", flush=True)
    rng = np.random.default_rng(B + I + O + dp)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    X, W, dY = from_vals(Xv, dtype), from_vals(Wv, dtype), from_vals(dYv, dtype)
    tm = P.tile_mask(O, I, x, y, dp, b)
    MW = P.expand_tile_mask(tm, O, I, x, y).astype(np.float64)
    ones = np.ones(O, np.uint8)
    pat = ard.Pattern.tile(dp, b, x, y)
    Y = torch.full((B, O), float("nan"), dtype=X.dtype, device="cuda")
    dX = torch.full((B, I), float("nan"), dtype=X.dtype, device="cuda")
    dW = torch.full((O, I), float("nan"), dtype=X.dtype, device="cuda")
    ard.drop_gemm_fwd(X, W, pat, alpha=0.5, out=Y)
    ard.drop_gemm_bwd_data(dY, W, pat, out=dX)
    ard.drop_gemm_bwd_weight(dY, X, pat, out=dW)
    assert_parity(Y, G.drop_gemm_fwd(Xv, Wv, MW, ones, 0.5), dtype, what="Y")
    assert_parity(dX, G.drop_gemm_bwd_data(dYv, Wv, MW, ones), dtype, what="dX")
    assert_parity(dW, G.drop_gemm_bwd_weight(dYv, Xv, MW, ones), dtype, zero_mask=(MW == 0), what="dW")
    # precomputed lists from pattern_gen give the same bits as the internally generated ones
    lists = ard.pattern_gen(pat, O, I)
    pat2 = ard.Pattern.tile(dp, b, x, y, lists=lists)
    Y2 = ard.drop_gemm_fwd(X, W, pat2, alpha=0.5)
    assert torch.equal(Y2.view(torch.int16 if dtype == "bf16" else torch.int32),
                       Y.view(torch.int16 if dtype == "bf16" else torch.int32))


def test_results_are_deterministic():
    rng = np.random.default_rng(3)
    X, W = from_vals(rng.standard_normal((300, 520)), "bf16"), from_vals(rng.standard_normal((260, 520)), "bf16")
    pat = ard.Pattern.row(3, 2)
    a = ard.drop_gemm_fwd(X, W, pat, ard.Pattern.row(2, 1))
    b = ard.drop_gemm_fwd(X, W, pat, ard.Pattern.row(2, 1))
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_relu_bwd_kernel():
    rng = np.random.default_rng(4)
    dYv, Yv = stored(rng.standard_normal(1000), "bf16"), stored(rng.standard_normal(1000), "bf16")
    out = ard.relu_bwd(from_vals(dYv, "bf16"), from_vals(Yv, "bf16"))
    assert_parity(out, G.relu_bwd(dYv, Yv), "bf16", zero_mask=(Yv <= 0), what="relu_bwd")
