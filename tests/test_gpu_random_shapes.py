"""GPU parity on seeded random layers: sizes, row patterns and layout flags drawn at random, every GEMM
entry point against the oracle.  Exercises the dispatch rules (tile choice, split contractions, scattering
epilogue, finishing pass, narrow layers) away from the benchmark shapes."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from paper_2203_05705_amd import binding as ard
from util import assert_parity, from_vals, raw_bits, stored

pytestmark = pytest.mark.gpu
IN, OUT, WC, DW = ard.IN_COMPACT, ard.OUT_COMPACT, ard.W_COMPACT, ard.DW_COMPACT


def draw_case(rng):
    big = rng.random() < 0.3
    B = int(rng.integers(1, 1500 if big else 300))
    I = int(rng.integers(1, 160 if big else 260)) * 8 + (int(rng.integers(0, 8)) if rng.random() < 0.4 else 0)
    O = int(rng.integers(1, 2100 if big else 600))
    if rng.random() < 0.25:
        O = int(rng.integers(1, 17))          # narrow layer
    po = pi = None
    if rng.random() < 0.7:
        dp = int(rng.integers(1, min(O, 8) + 1))
        po = (dp, int(rng.integers(1, dp + 1)))
    if rng.random() < 0.7:
        dp = int(rng.integers(1, min(I, 8) + 1))
        pi = (dp, int(rng.integers(1, dp + 1)))
    return B, I, O, po, pi


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("seed", range(6))
def test_random_layers(seed, dtype):
    rng = np.random.default_rng(1000 + seed)
    for case in range(5):
        B, I, O, po, pi = draw_case(rng)
        print(f"{dtype} seed {seed} case {case}: B={B} I={I} O={O} pat_out={po} pat_in={pi}", flush=True)
        Xv, Wv, dYv = (stored(rng.standard_normal(s) * 0.5, dtype) for s in ((B, I), (O, I), (B, O)))
        mo = P.row_mask(O, *po) if po else np.ones(O, np.uint8)
        mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
        ko, ki = P.keep_list(mo), P.keep_list(mi)
        MW = G.weight_mask_rows(mo, mi)
        pat_o = ard.Pattern.row(*po) if po else None
        pat_i = ard.Pattern.row(*pi) if pi else None
        refY = G.drop_gemm_fwd(Xv, Wv, MW, mo, 1.0, relu=True)
        refdX = G.drop_gemm_bwd_data(dYv, Wv, MW, mo, 1.0)
        refdW = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo)
        X, W, dY = (from_vals(v, dtype) for v in (Xv, Wv, dYv))
        Xc, dYc = ard.pad_compact(from_vals(Xv[:, ki], dtype)), ard.pad_compact(from_vals(dYv[:, ko], dtype))
        Wc = ard.compact_weight(W, pat_o, pat_i)
        zo, zi = (mo == 0)[None, :], (mi == 0)[None, :]
        assert_parity(ard.drop_gemm_fwd(X, W, pat_o, pat_i, relu=True), refY, dtype, zero_mask=zo, what="Y")
        assert_parity(ard.drop_gemm_bwd_data(dY, W, pat_o, pat_i), refdX, dtype, zero_mask=zi, what="dX")
        assert_parity(ard.drop_gemm_bwd_weight(dY, X, pat_o, pat_i), refdW, dtype, zero_mask=(MW == 0), what="dW")
        for flags, Wt in ((IN | OUT, W), (IN | OUT | WC, Wc), (IN, W), (OUT, W)):
            Xin, dYin = (Xc if flags & IN else X), (dYc if flags & OUT else dY)
            Y = ard.drop_gemm_fwd(Xin, Wt, pat_o, pat_i, relu=True, flags=flags, I=I, O=O)
            if flags & OUT:
                assert_parity(Y[:, :len(ko)].contiguous(), refY[:, ko], dtype, what=f"Y flags={flags}")
                assert not raw_bits(Y[:, len(ko):].contiguous()).any(), "Y padding"
            else:
                assert_parity(Y, refY, dtype, zero_mask=zo, what=f"Y flags={flags}")
            dX = ard.drop_gemm_bwd_data(dYin, Wt, pat_o, pat_i, flags=flags, I=I, O=O)
            if flags & IN:
                assert_parity(dX[:, :len(ki)].contiguous(), refdX[:, ki], dtype, what=f"dX flags={flags}")
                assert not raw_bits(dX[:, len(ki):].contiguous()).any(), "dX padding"
            else:
                assert_parity(dX, refdX, dtype, zero_mask=zi, what=f"dX flags={flags}")
            if not flags & WC:
                dW = torch.full((O, I), float("nan"), dtype=X.dtype, device="cuda")
                ard.drop_gemm_bwd_weight(dYin, Xin, pat_o, pat_i, flags=flags, out=dW, I=I, O=O)
                assert_parity(dW, refdW, dtype, zero_mask=(MW == 0), what=f"dW flags={flags}")
        dWc = ard.drop_gemm_bwd_weight(dYc, Xc, pat_o, pat_i, flags=IN | OUT | DW, I=I, O=O)
        assert_parity(dWc[:len(ko), :len(ki)].contiguous(), refdW[np.ix_(ko, ki)], dtype, what="dW compact")
        bits = raw_bits(dWc)
        assert not bits[len(ko):, :].any() and not bits[:, len(ki):].any(), "dW compact padding"


def draw_tile_case(rng):
    B = int(rng.integers(100, 330)) * 8 + (int(rng.integers(0, 8)) if rng.random() < 0.3 else 0)
    I = int(rng.integers(100, 520)) * 8
    O = int(rng.integers(100, 330)) * 8
    x, y = int(rng.choice([32, 64, 128, 256])), int(rng.choice([32, 64, 128, 256]))
    dp = int(rng.integers(1, 9))
    b = int(rng.integers(1, dp + 1))
    return B, I, O, x, y, dp, b


@pytest.mark.parametrize("seed", range(8))
def test_random_tile_patterns(seed):
    """Tile patterns at sizes that take the class-grouped large-tile kernels: random tile shapes, periods
    and extents that end inside their last tile row / column."""
    from test_gpu_fast import _tile_case
    rng = np.random.default_rng(2000 + seed)
    B, I, O, x, y, dp, b = draw_tile_case(rng)
    print(f"seed {seed}: B={B} I={I} O={O} tile {x}x{y} dp={dp} b={b}", flush=True)
    Xv, Wv, dYv = (stored(rng.standard_normal(s) * 0.5, "bf16") for s in ((B, I), (O, I), (B, O)))
    _tile_case(Xv, Wv, dYv, from_vals(Xv, "bf16"), from_vals(Wv, "bf16"), from_vals(dYv, "bf16"), x, y, dp, b, f"seed {seed}")
