"""GPU parity: pattern_gen masks and index lists must be bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from oracle import patterns as P
from paper_2203_05705_amd import binding as ard

pytestmark = pytest.mark.gpu


def _np(t):
    return t.cpu().numpy()


ROW_CASES = [(1, 1, 1), (7, 3, 2), (64, 1, 1), (64, 64, 64), (1024, 2, 1), (1024, 2, 2), (2048, 3, 1), (2048, 3, 3),
             (2048, 5, 4), (2048, 8, 8), (1000, 7, 5), (4097, 6, 2), (100000, 9, 9), (1025, 1024, 1000)]


@pytest.mark.parametrize("n,dp,b", ROW_CASES)
def test_row_pattern_bit_exact(n, dp, b):
    print(f"row pattern n={n} dp={dp} b={b}", flush=True)
    out = ard.pattern_gen(ard.Pattern.row(dp, b), n)
    torch.cuda.synchronize()
    m = P.row_mask(n, dp, b)
    keep = P.keep_list(m)
    assert np.array_equal(_np(out["mask"]), m)
    cnt = int(out["count"].item())
    assert cnt == len(keep)
    assert np.array_equal(_np(out["keep"])[:cnt], keep)
    assert np.all(_np(out["keep"])[cnt:] == -1)            # nothing written past the kept count


TILE_CASES = [(64, 64, 32, 32, 2, 1), (4096, 4096, 64, 64, 2, 1), (4096, 4096, 64, 64, 3, 2), (4096, 4096, 64, 64, 4, 4),
              (4096, 4096, 64, 64, 7, 3), (4096, 4096, 32, 32, 5, 5), (100, 70, 32, 32, 3, 1), (2048, 784, 64, 64, 3, 3),
              (130, 4100, 64, 32, 8, 6), (65, 33, 16, 8, 11, 7), (4096, 4096, 64, 64, 1, 1), (128, 128, 64, 64, 4, 2)]


@pytest.mark.parametrize("O,I,x,y,dp,b", TILE_CASES)
def test_tile_pattern_bit_exact(O, I, x, y, dp, b):
    print(f"tile pattern O={O} I={I} tile={x}x{y} dp={dp} b={b}", flush=True)
    out = ard.pattern_gen(ard.Pattern.tile(dp, b, x, y), O, I)
    torch.cuda.synchronize()
    tm = P.tile_mask(O, I, x, y, dp, b)
    keep = P.keep_list(tm)
    rowptr, _ = P.tile_csr(tm)
    colptr, rows = P.tile_csc(tm)
    cnt = int(out["count"].item())
    assert cnt == len(keep)
    assert np.array_equal(_np(out["mask"]), tm.reshape(-1))
    assert np.array_equal(_np(out["keep"])[:cnt], keep)
    assert np.array_equal(_np(out["rowptr"]), rowptr)
    assert np.array_equal(_np(out["colptr"]), colptr)
    assert np.array_equal(_np(out["csc_rows"])[:cnt], rows)
    assert np.all(_np(out["keep"])[cnt:] == -1) and np.all(_np(out["csc_rows"])[cnt:] == -1)


def test_sampled_patterns_of_100_iterations_bit_exact():
    """Config 2: a new (dp, b) per iteration and layer from the searched distribution."""
    from oracle import sampler as S
    from oracle import search as K
    for p in (0.3, 0.5, 0.7):
        d, _ = K.search_k(p, 8)
        cdf = [int(c) for c in K.fixed_point_cdf(d)]
        for it in range(100):
            for layer in (1, 2):
                dp, b = ard.pattern_sample(cdf, 2, it, layer)
                assert (dp, b) == S.sample_pattern(cdf, 2, it, layer)
                if it % 10 == 0:
                    out = ard.pattern_gen(ard.Pattern.row(dp, b), 2048)
                    m = P.row_mask(2048, dp, b)
                    assert np.array_equal(_np(out["mask"]), m)
                    cnt = int(out["count"].item())
                    assert np.array_equal(_np(out["keep"])[:cnt], P.keep_list(m))
