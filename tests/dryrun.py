"""Raw-ctypes calls of the library in dry-run mode: argument checks, dispatch and the host-side bounds
proof of the loaders run, nothing is launched, device pointers are fake.  Works without a GPU."""
import ctypes as C
from contextlib import contextmanager

from paper_2203_05705_amd import binding as ard

BF16, F32 = ard.BF16, ard.F32


class FakeHeap:
    """Hands out distinct, 256-byte aligned fake device addresses."""

    def __init__(self):
        self.top = 0x7F0000000000

    def __call__(self, nbytes):
        p = self.top
        self.top += (int(nbytes) + 4095) // 256 * 256
        return p


@contextmanager
def dry_run():
    lib = ard.lib()
    lib.ard_debug_set_dry_run(1)
    try:
        yield lib
    finally:
        lib.ard_debug_set_dry_run(0)
        lib.ard_debug_set_extent_slack(0)


def launches(lib):
    buf = C.create_string_buffer(2048)
    n = lib.ard_debug_dry_launches(buf, 2048)
    return n, buf.value.decode().split(",") if buf.value else []


def last_bounds(lib):
    six = (C.c_int64 * 6)()
    n = lib.ard_debug_last_bounds(six)
    return n, list(six)


def cpat(p, kind=ard.PAT_ROW, tile=(0, 0)):
    if p is None:
        return None, None
    s = ard.CPattern(kind, p[0], p[1], tile[0], tile[1], 0, None, None, None, None, None)
    return s, C.byref(s)


def layer_calls(lib, heap, dtype, B, I, O, po, pi, flags, tile=None, ws_bytes=1 << 28, ops=(0, 1, 2)):
    """Issues fwd / bwd_data / bwd_weight of one layer; returns the list of status codes."""
    es = 2 if dtype == BF16 else 4
    if tile:
        so, ro = cpat(po, ard.PAT_TILE, tile)
        si, ri = None, None
    else:
        so, ro = cpat(po)
        si, ri = cpat(pi)
    big = max(B, 8) * (max(I, O) + 8) * es + (O + 8) * (I + 8) * es
    X, W, Y, dY, dX, dW, src = (heap(big) for _ in range(7))
    ws = heap(ws_bytes)
    rc = []
    if 0 in ops:
        rc.append(lib.ard_drop_gemm_fwd(dtype, B, I, O, X, W, Y, ro, ri, 1.0, 1, flags & ~ard.DW_COMPACT, ws, ws_bytes, None))
    if 1 in ops:
        rc.append(lib.ard_drop_gemm_bwd_data(dtype, B, I, O, dY, W, dX, ro, ri, 1.0, src, flags & ~ard.DW_COMPACT, ws,
                                             ws_bytes, None))
    if 2 in ops:
        rc.append(lib.ard_drop_gemm_bwd_weight(dtype, B, I, O, dY, X, dW, ro, ri, 1.0, 0.0, flags & ~ard.W_COMPACT, ws,
                                               ws_bytes, None))
    return rc


def lstm_calls(lib, heap, dtype, T, B, I, H, pat):
    s, r = cpat(pat)
    es = 2 if dtype == BF16 else 4
    n = lib.ard_lstm_workspace_bytes(dtype, T, B, I, H, r)
    ws = heap(n)
    x, W, h, c, g, dh, dx, dW = (heap(T * B * (4 * H + I) * 4 + 4 * H * (I + H) * es) for _ in range(8))
    return [lib.ard_lstm_fwd(dtype, T, B, I, H, x, W, r, h, c, g, ws, n, None),
            lib.ard_lstm_bwd(dtype, T, B, I, H, x, W, r, h, c, g, dh, dx, dW, ws, n, None)]


def conv_calls(lib, heap, dtype, N, Cc, Cout, H, W, k, stride, pad, n_keep, modes=(1, 2, 3, 0x101, 0x202, 0x103)):
    n = lib.ard_conv_workspace_bytes(dtype, N, Cc, H, W, Cout, k, k, stride, pad)
    ws = heap(n)
    big = N * max(Cc, Cout) * (H + 2 * pad) * (W + 2 * pad) * 4
    A, Wt, dY, out, keep, mask = (heap(big) for _ in range(6))
    return [lib.ard_fmap_drop_conv(m, dtype, N, Cc, H, W, Cout, k, k, stride, pad, 0.0, n_keep, A, Wt, dY, out,
                                   mask, keep, None, None, ws, n, None) for m in modes]
