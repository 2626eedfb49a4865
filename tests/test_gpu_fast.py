"""GPU parity at sizes that take the large-tile (256x256, class-grouped) path, including
BASELINE config 3 (4096^3 bf16, 64x64 tiles) in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from paper_2203_05705_amd import binding as ard
from paper_2203_05705_amd import workloads as WL
from util import assert_parity, from_vals, stored, to_dev

pytestmark = pytest.mark.gpu


def _tile_case(Xv, Wv, dYv, X, W, dY, x, y, dp, b, what):
    B, I = Xv.shape
    O = Wv.shape[0]
    tm = P.tile_mask(O, I, x, y, dp, b)
    MW = P.expand_tile_mask(tm, O, I, x, y).astype(np.float64)
    ones = np.ones(O, np.uint8)
    pat = ard.Pattern.tile(dp, b, x, y)
    Y = torch.full((B, O), float("nan"), dtype=X.dtype, device="cuda")
    dX = torch.full((B, I), float("nan"), dtype=X.dtype, device="cuda")
    dW = torch.full((O, I), float("nan"), dtype=X.dtype, device="cuda")
    ard.drop_gemm_fwd(X, W, pat, out=Y)
    ard.drop_gemm_bwd_data(dY, W, pat, out=dX)
    ard.drop_gemm_bwd_weight(dY, X, pat, out=dW)
    torch.cuda.synchronize()
    e = [assert_parity(Y, G.drop_gemm_fwd(Xv, Wv, MW, ones), "bf16", what=what + " Y"),
         assert_parity(dX, G.drop_gemm_bwd_data(dYv, Wv, MW, ones), "bf16", what=what + " dX"),
         assert_parity(dW, G.drop_gemm_bwd_weight(dYv, Xv, MW, ones), "bf16", zero_mask=(MW == 0), what=what + " dW")]
    print(what, "max rel err", ["%.2e" % v for v in e], flush=True)


@pytest.mark.parametrize("dp,b", [(2, 1), (3, 2), (4, 4), (1, 1), (5, 3), (6, 2), (7, 7), (8, 5)])
def test_config3_tile_gemm_full_size(dp, b):
    """W 4096x4096 ~N(0,0.02), X 4096x4096 ~N(0,1), 64x64 tiles; every output element checked."""
    wl = WL.tile_gemm(seed=3)
    Xv, Wv, dYv = wl.values("X"), wl.values("W"), wl.values("dY")
    X, W, dY = (to_dev(wl.arrays[k], "bf16") for k in ("X", "W", "dY"))
    print(f"config 3 dp={dp} b={b}", flush=True)
    _tile_case(Xv, Wv, dYv, X, W, dY, 64, 64, dp, b, f"config3 dp={dp}")


@pytest.mark.parametrize("B,I,O,x,y,dp,b", [
    (2304, 2112, 2240, 64, 64, 3, 1),      # ragged: clipped edge tiles, partial row/column groups
    (2048, 2048, 4096, 128, 64, 7, 5),
    (2048, 2048, 2048, 32, 64, 3, 2),      # 32-row tiles
    (2050, 2056, 2312, 64, 128, 6, 4),     # gcd(TC, dp) > 1 and ragged batch
    (2048, 4096, 4096, 256, 256, 2, 2),
    (2048, 5128, 2048, 64, 128, 2, 1),     # long contraction whose last 128-wide block holds 8 columns (kept)
    (2048, 5128, 2048, 64, 128, 2, 2),     # ... (dropped)
    (1965, 2760, 2480, 256, 64, 7, 1),     # W ends 176 rows into its last 256-row tile row (loaders clamp there)
    (968, 1864, 3144, 256, 128, 3, 3),     # both axes end inside their last block
])
def test_large_tile_path_other_shapes(B, I, O, x, y, dp, b):
    print(f"large tile case B={B} I={I} O={O} tile={x}x{y} dp={dp} b={b}", flush=True)
    rng = np.random.default_rng(B + O + dp)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), "bf16") for s in ((B, I), (O, I), (B, O)))
    _tile_case(Xv, Wv, dYv, from_vals(Xv, "bf16"), from_vals(Wv, "bf16"), from_vals(dYv, "bf16"), x, y, dp, b, "large")


@pytest.mark.parametrize("B,I,O,x,y,dp,b", [
    (2048, 2048, 2048, 32, 32, 2, 1),      # the tile size of Section 3.2: two kept 32-wide blocks per 64-deep step
    (1024, 2048, 2048, 32, 32, 3, 3),      # kept-block counts of both parities over the classes
    (512, 784, 2048, 32, 32, 3, 1),        # input width ends 16 columns into its last tile column
    (512, 1024, 1000, 32, 32, 2, 2),       # output width ends 8 rows into its last tile row
    (1030, 1096, 1192, 32, 32, 7, 4),      # everything ragged
    (2048, 2048, 2048, 64, 32, 5, 2),
    (2048, 2048, 2048, 32, 128, 4, 3),
])
def test_large_tile_path_32_wide_tiles(B, I, O, x, y, dp, b):
    print(f"32-wide tile case B={B} I={I} O={O} tile={x}x{y} dp={dp} b={b}", flush=True)
    rng = np.random.default_rng(B + O + dp + 32)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), "bf16") for s in ((B, I), (O, I), (B, O)))
    _tile_case(Xv, Wv, dYv, from_vals(Xv, "bf16"), from_vals(Wv, "bf16"), from_vals(dYv, "bf16"), x, y, dp, b, "tile32")


def test_tile_pattern_data_gradient_with_fused_relu_gradient():
    """dX gated by the sign of a second matrix in the epilogue of the tile-class product."""
    B, I, O, x, y, dp, b = 1024, 2048, 2048, 32, 32, 3, 2
    rng = np.random.default_rng(99)
    Wv, dYv, src = (stored(rng.standard_normal(s), "bf16") for s in ((O, I), (B, O), (B, I)))
    MW = P.expand_tile_mask(P.tile_mask(O, I, x, y, dp, b), O, I, x, y).astype(np.float64)
    dX = torch.full((B, I), float("nan"), dtype=torch.bfloat16, device="cuda")
    ard.drop_gemm_bwd_data(from_vals(dYv, "bf16"), from_vals(Wv, "bf16"), ard.Pattern.tile(dp, b, x, y),
                           relu_src=from_vals(src, "bf16"), out=dX)
    ref = G.relu_bwd(G.drop_gemm_bwd_data(dYv, Wv, MW, np.ones(O, np.uint8)), src)
    assert_parity(dX, ref, "bf16", zero_mask=(src <= 0), what="tile dX relu")


@pytest.mark.parametrize("B,I,O", [(4096, 2048, 4096), (4000, 2056, 4104)])
def test_large_dense_path(B, I, O):
    """Rate 0 (no pattern) through the large-tile kernels, all three products."""
    print(f"large dense case B={B} I={I} O={O}", flush=True)
    rng = np.random.default_rng(B + I)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), "bf16") for s in ((B, I), (O, I), (B, O)))
    X, W, dY = from_vals(Xv, "bf16"), from_vals(Wv, "bf16"), from_vals(dYv, "bf16")
    ones_o = np.ones(O, np.uint8)
    MW = np.ones((O, I))
    assert_parity(ard.drop_gemm_fwd(X, W, relu=True), G.drop_gemm_fwd(Xv, Wv, MW, ones_o, relu=True), "bf16", what="Y")
    assert_parity(ard.drop_gemm_bwd_data(dY, W, alpha=0.5), G.drop_gemm_bwd_data(dYv, Wv, MW, ones_o, 0.5), "bf16", what="dX")
    assert_parity(ard.drop_gemm_bwd_weight(dY, X), G.drop_gemm_bwd_weight(dYv, Xv, MW, ones_o), "bf16", what="dW")
