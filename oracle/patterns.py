"""Dropout patterns as explicit 0/1 masks (test oracle, CPU only).

Row-based pattern: Section 3.1, Eq. (1).  Tile-based pattern: Section 3.2.
Mask convention (Section 6, the "1,0,1,1,0,0" example): 1 = kept, 0 = dropped.

Indexing: the paper numbers rows/tiles from 1 and takes the bias b in {1..dp};
a unit with 1-based index i is DROPPED iff (i - b) mod dp != 0.  The worked
example dp=3, b=1 therefore keeps units 1, 4, 7, ...
"""
import numpy as np


def check_params(dp: int, b: int, n_units: int) -> None:
    """dp ranges over 1..(number of units) (Sections 3.1/3.2, dp_max); b over 1..dp."""
    if not (1 <= dp <= max(1, n_units)):
        raise ValueError(f"dp={dp} outside 1..{n_units}")
    if not (1 <= b <= dp):
        raise ValueError(f"b={b} outside 1..{dp}")


def row_mask(n: int, dp: int, b: int) -> np.ndarray:
    """Eq. (1) over n units; returns uint8[n] with 1 = kept."""
    check_params(dp, b, n)
    m = np.zeros(n, dtype=np.uint8)
    for i in range(1, n + 1):            # the paper's 1-based index
        if (i - b) % dp == 0:
            m[i - 1] = 1
    return m


def tile_grid(O: int, I: int, tile_r: int, tile_c: int):
    """Number of tile rows / columns covering W[O x I]; edge tiles are clipped."""
    return -(-O // tile_r), -(-I // tile_c)


def tile_mask(O: int, I: int, tile_r: int, tile_c: int, dp: int, b: int) -> np.ndarray:
    """Eq. (1) applied to the 1-based row-major linear index of the tile grid
    over W[O x I] (Section 3.2: dp-1 of every dp successive tiles are dropped).
    Returns uint8[TR, TC], 1 = kept."""
    TR, TC = tile_grid(O, I, tile_r, tile_c)
    check_params(dp, b, TR * TC)
    m = np.zeros((TR, TC), dtype=np.uint8)
    for tr in range(TR):
        for tc in range(TC):
            i = tr * TC + tc + 1
            if (i - b) % dp == 0:
                m[tr, tc] = 1
    return m


def expand_tile_mask(tm: np.ndarray, O: int, I: int, tile_r: int, tile_c: int) -> np.ndarray:
    """Element mask uint8[O, I] of a tile mask (every synapse of a dropped tile is dropped)."""
    full = np.repeat(np.repeat(tm, tile_r, axis=0), tile_c, axis=1)
    return np.ascontiguousarray(full[:O, :I])


def keep_list(mask: np.ndarray) -> np.ndarray:
    """Ascending indices of kept units of a flat mask (int32)."""
    return np.flatnonzero(mask.reshape(-1)).astype(np.int32)


def tile_csr(tm: np.ndarray):
    """Per tile-row lists of kept tile columns: (rowptr int32[TR+1], cols int32[nnz])."""
    TR, TC = tm.shape
    rowptr = np.zeros(TR + 1, dtype=np.int32)
    cols = []
    for tr in range(TR):
        for tc in range(TC):
            if tm[tr, tc]:
                cols.append(tc)
        rowptr[tr + 1] = len(cols)
    return rowptr, np.asarray(cols, dtype=np.int32)


def tile_csc(tm: np.ndarray):
    """Per tile-column lists of kept tile rows: (colptr int32[TC+1], rows int32[nnz])."""
    TR, TC = tm.shape
    colptr = np.zeros(TC + 1, dtype=np.int32)
    rows = []
    for tc in range(TC):
        for tr in range(TR):
            if tm[tr, tc]:
                rows.append(tr)
        colptr[tc + 1] = len(rows)
    return colptr, np.asarray(rows, dtype=np.int32)
