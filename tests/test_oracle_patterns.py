"""Pins for the oracle's pattern definitions (Sections 3.1, 3.2, 6)."""
import json
import os

import numpy as np
import pytest

from oracle import patterns as P


@pytest.fixture(scope="module")
def golden(golden_dir):
    with open(os.path.join(golden_dir, "paper_examples.json")) as f:
        return json.load(f)


def test_row_example_from_paper(golden):
    g = golden["row_dp3_b1"]
    m = P.row_mask(g["n"], g["dp"], g["b"])
    assert (P.keep_list(m) + 1).tolist() == g["kept_1based"]


def test_tile_example_from_paper(golden):
    g = golden["tile_dp4_b1"]
    TR, TC = g["grid"]
    tm = P.tile_mask(TR * 32, TC * 32, 32, 32, g["dp"], g["b"])
    assert (P.keep_list(tm) + 1).tolist() == g["kept_1based"]
    assert tm.mean() == g["kept_fraction"]
    full = P.expand_tile_mask(tm, TR * 32, TC * 32, 32, 32)
    assert full.mean() == g["kept_fraction"]          # 1/4 of the synapses survive


def test_mask_polarity_from_paper(golden):
    g = golden["cnn_row_mask"]
    m = np.ones(6, dtype=np.uint8)
    for i in g["dropped_1based"]:
        m[i - 1] = 0
    assert m.tolist() == g["mask"]
    # the oracle's masks use the same polarity: kept list = positions of ones
    assert P.keep_list(m).tolist() == [0, 2, 3]


def test_half_kept_at_dp2(golden):
    for b in (1, 2):
        assert P.row_mask(1024, 2, b).mean() == golden["row_dp2"]["kept_fraction"]


@pytest.mark.parametrize("n", [1, 2, 7, 16, 63, 64])
def test_row_mask_all_patterns_bruteforce(n):
    for dp in range(1, n + 1):
        union = np.zeros(n, dtype=np.int64)
        for b in range(1, dp + 1):
            m = P.row_mask(n, dp, b)
            # independent formulation: kept 0-based rows are b-1, b-1+dp, ...
            ref = np.zeros(n, dtype=np.uint8)
            ref[list(range(b - 1, n, dp))] = 1
            assert np.array_equal(m, ref)
            assert int(m.sum()) == -(-(n - (b - 1)) // dp) if n > b - 1 else int(m.sum()) == 0
            union += m
        assert np.all(union == 1)                      # every row is kept by exactly one bias


def test_row_mask_counts_at_benchmark_sizes():
    assert [int(P.row_mask(2048, 3, b).sum()) for b in (1, 2, 3)] == [683, 683, 682]
    assert [int(P.row_mask(2048, 5, b).sum()) for b in range(1, 6)] == [410, 410, 410, 409, 409]
    assert int(P.row_mask(1024, 2, 1).sum()) == 512


def test_param_validation():
    with pytest.raises(ValueError):
        P.row_mask(8, 0, 1)
    with pytest.raises(ValueError):
        P.row_mask(8, 3, 4)
    with pytest.raises(ValueError):
        P.row_mask(8, 3, 0)
    with pytest.raises(ValueError):
        P.row_mask(8, 9, 1)                             # dp_max = number of rows
    with pytest.raises(ValueError):
        P.tile_mask(64, 64, 32, 32, 5, 1)               # dp_max = number of tiles


@pytest.mark.parametrize("O,I,x,y", [(64, 64, 32, 32), (100, 70, 32, 32), (256, 192, 64, 64), (65, 33, 16, 8)])
def test_tile_mask_partition_and_lists(O, I, x, y):
    TR, TC = P.tile_grid(O, I, x, y)
    assert TR == -(-O // x) and TC == -(-I // y)
    for dp in range(1, min(TR * TC, 9) + 1):
        union = np.zeros((TR, TC), dtype=np.int64)
        for b in range(1, dp + 1):
            tm = P.tile_mask(O, I, x, y, dp, b)
            lin = np.arange(TR * TC)
            assert np.array_equal(tm.reshape(-1), ((lin - (b - 1)) % dp == 0).astype(np.uint8))
            union += tm
            rowptr, cols = P.tile_csr(tm)
            colptr, rows = P.tile_csc(tm)
            nnz = int(tm.sum())
            assert rowptr[-1] == nnz == colptr[-1] == len(cols) == len(rows)
            csr_pairs = {(tr, int(c)) for tr in range(TR) for c in cols[rowptr[tr]:rowptr[tr + 1]]}
            csc_pairs = {(int(r), tc) for tc in range(TC) for r in rows[colptr[tc]:colptr[tc + 1]]}
            assert csr_pairs == csc_pairs == {(int(t) // TC, int(t) % TC) for t in P.keep_list(tm)}
            for tr in range(TR):
                seg = cols[rowptr[tr]:rowptr[tr + 1]]
                assert np.all(np.diff(seg) > 0)
            full = P.expand_tile_mask(tm, O, I, x, y)
            assert full.shape == (O, I)
            for (o, i) in [(0, 0), (O - 1, I - 1), (O // 2, I // 3)]:
                assert full[o, i] == tm[o // x, i // y]
        assert np.all(union == 1)


def test_tile_columns_when_grid_width_divisible():
    # 64x64 grid (4096/64): dp | TC makes kept tiles whole tile columns; dp=3 gives diagonals
    tm = P.tile_mask(4096, 4096, 64, 64, 2, 1)
    assert np.all(tm[:, 0::2] == 1) and np.all(tm[:, 1::2] == 0)
    tm3 = P.tile_mask(4096, 4096, 64, 64, 3, 1)
    assert sorted(set(tm3.sum(axis=1).tolist())) == [21, 22]
    assert int(tm3.sum()) == 1366
