"""Host-side bounds proof of the LDS-direct loaders, without a GPU.

In dry-run mode every entry point runs its dispatch and, for each launch that fetches operands with
unchecked per-lane addresses, walks every workgroup, wavefront, lane and contraction step with the
kernel's own address arithmetic and checks the bytes touched against the operand's extent.  These
tests push the benchmark configurations and the seeded random generators of the GPU tests through it."""
import numpy as np
import pytest

import dryrun as D
from paper_2203_05705_amd import binding as ard

IN, OUT, WC, DW = ard.IN_COMPACT, ard.OUT_COMPACT, ard.W_COMPACT, ard.DW_COMPACT


def _ok(lib, rcs, what):
    for rc in rcs:
        assert rc == 0, f"{what}: status {rc}: {lib.ard_last_error().decode()}"


def test_dry_run_launches_nothing_and_reports_kernels():
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 2048, (2, 1), (2, 2), IN | OUT), "layer")
        n, names = D.launches(lib)
        assert n >= 3 and "gemm_direct_kernel" in names
        n_proofs, six = D.last_bounds(lib)
        assert n_proofs >= 3
        a_lo, a_hi, a_bytes, b_lo, b_hi, b_bytes = six
        assert 0 <= a_lo < a_hi <= a_bytes and 0 <= b_lo < b_hi <= b_bytes


def test_config2_all_pattern_pairs():
    """MLP 784-2048-2048-10 at batch 1024: the nine calls of an iteration for all 64 (dp1, dp2)."""
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        proofs = 0
        for dp1 in range(1, 9):
            for dp2 in range(1, 9):
                p1, p2 = (dp1, 1 + (dp1 * 3 + dp2) % dp1), (dp2, 1 + (dp1 + dp2 * 5) % dp2)
                w = f"pair {p1} {p2}"
                _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 784, 2048, p1, None, OUT, ops=(0, 2)), w + " L1")
                _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 2048, p2, p1, IN | OUT), w + " L2")
                _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 2048, p2, p1, IN | OUT | WC, ops=(0, 1)), w + " L2c")
                _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 10, None, p2, IN | OUT), w + " L3")
                proofs += D.last_bounds(lib)[0]
        assert proofs >= 64 * 5


@pytest.mark.parametrize("dp", range(1, 9))
def test_config3_tile_patterns(dp):
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        for b in range(1, dp + 1):
            _ok(lib, D.layer_calls(lib, heap, D.BF16, 4096, 4096, 4096, (dp, b), None, 0, tile=(64, 64)), f"dp={dp} b={b}")
        assert D.last_bounds(lib)[0] >= 1


def test_random_layers_and_tile_patterns():
    from test_gpu_random_shapes import draw_case, draw_tile_case
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        for seed in range(40):
            rng = np.random.default_rng(1000 + seed)
            for _ in range(5):
                B, I, O, po, pi = draw_case(rng)
                for flags in (0, IN | OUT, IN | OUT | WC, IN, OUT, IN | OUT | DW):
                    _ok(lib, D.layer_calls(lib, heap, D.BF16, B, I, O, po, pi, flags), f"layer {B} {I} {O} {po} {pi} {flags}")
        for seed in range(60):
            B, I, O, x, y, dp, b = draw_tile_case(np.random.default_rng(2000 + seed))
            _ok(lib, D.layer_calls(lib, heap, D.BF16, B, I, O, (dp, b), None, 0, tile=(x, y)), f"tile {B} {I} {O} {x}x{y} {dp},{b}")
        assert D.last_bounds(lib)[0] > 100


def test_the_shape_that_faulted_once():
    """W 2480 x 2760 with 256-row tiles: the last tile row holds 176 rows (block axes are clamped)."""
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 1965, 2760, 2480, (7, 1), None, 0, tile=(256, 64)), "256x64")
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 968, 1864, 3144, (3, 3), None, 0, tile=(256, 128)), "256x128")


def test_lstm_and_conv_shapes():
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        for T, B, I, H, dp, b in [(64, 128, 1024, 1024, 2, 2), (64, 128, 1024, 1024, 1, 1), (64, 128, 1024, 1024, 3, 1),
                                  (5, 6, 24, 32, 2, 1), (4, 3, 10, 37, 3, 3), (3, 70, 40, 64, 1, 1), (6, 33, 72, 136, 4, 2),
                                  (3, 64, 128, 200, 3, 1), (35, 20, 1500, 1500, 2, 1)]:
            _ok(lib, D.lstm_calls(lib, heap, D.BF16, T, B, I, H, (dp, b)), f"lstm {T} {B} {I} {H} {dp}")
        n_lstm = D.last_bounds(lib)[0]
        for N, Cc, Cout, H, W, k, pad, nk in [(128, 256, 256, 28, 28, 3, 1, 128), (128, 256, 256, 28, 28, 3, 1, 256),
                                              (2, 8, 16, 7, 7, 3, 1, 4), (3, 12, 20, 9, 6, 3, 1, 8), (2, 16, 8, 8, 8, 1, 0, 12),
                                              (2, 6, 10, 11, 10, 5, 2, 3), (5, 24, 130, 10, 12, 3, 1, 6), (7, 70, 300, 13, 17, 3, 1, 65),
                                              (3, 16, 24, 12, 12, 3, 0, 8), (2, 8, 8, 9, 7, 5, 1, 8),
                                              # few output positions: small tiles for many output channels
                                              (128, 512, 512, 7, 7, 3, 1, 256), (128, 512, 512, 14, 14, 3, 1, 256),
                                              (4, 64, 300, 7, 7, 3, 1, 64), (64, 128, 128, 56, 56, 3, 1, 64)]:
            modes = (1, 2, 3, 0x101, 0x202, 0x103) + ((0x303,) if k - 1 == 2 * pad else ())   # with and without shared grids
            _ok(lib, D.conv_calls(lib, heap, D.BF16, N, Cc, Cout, H, W, k, 1, pad, nk, modes=modes), f"conv {N} {Cc} {Cout} {H}x{W} k{k} keep {nk}")
        assert n_lstm >= 10 and D.last_bounds(lib)[0] >= 10 * 3
        # forward over a list of kept output positions (row-based sensitivity-aware pattern): the list lives in
        # device memory, the proof takes its two extreme readings
        for N, Cc, Cout, H, W, k, pad, rows_kept in [(128, 256, 256, 28, 28, 3, 1, 50000), (2, 8, 16, 7, 7, 3, 1, 40),
                                                       (5, 24, 130, 10, 12, 3, 1, 1), (3, 12, 20, 9, 6, 3, 1, 162)]:
            _ok(lib, D.conv_calls(lib, heap, D.BF16, N, Cc, Cout, H, W, k, 1, pad, rows_kept, modes=(4,)), f"rows {N} {Cc} {H}x{W}")
        assert D.last_bounds(lib)[0] == 4


def test_block_pattern_dispatch_and_bounds():
    """Forward pass under the block pattern: blocks of whole 64-channel groups over all taps with bands of at
    least half a tile go to the LDS-direct kernel (tile plan in the copy's launch, per-tile block lists, proof
    over the whole contraction); any other block shape goes to the general engine."""
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        for (N, Cc, Cout, H, W, k, pad, x, y), fast in [((128, 256, 256, 28, 28, 3, 1, 112, 576), True),
                                                         ((128, 256, 256, 28, 28, 3, 1, 196, 1152), True),
                                                         ((2, 128, 200, 12, 12, 3, 1, 72, 576), True),
                                                         ((3, 100, 140, 12, 13, 3, 1, 78, 576), True),
                                                         ((3, 100, 100, 12, 13, 3, 1, 156, 576), True),
                                                         ((2, 192, 130, 9, 16, 3, 1, 144, 0), True),
                                                         ((2, 128, 64, 12, 12, 3, 1, 72, 576), False),     # too few output channels
                                                         ((128, 256, 256, 28, 28, 3, 1, 8, 576), False),   # bands far below a tile
                                                         ((128, 256, 256, 28, 28, 3, 1, 112, 64), False),  # blocks cut channels
                                                         ((2, 128, 200, 12, 12, 3, 2, 18, 576), False)]:   # stride 2
            stride = 2 if (pad == 2) else 1
            pad = 1 if stride == 2 else pad
            n = lib.ard_conv_workspace_bytes(D.BF16, N, Cc, H, W, Cout, k, k, stride, pad)
            ws = heap(n)
            big = N * max(Cc, Cout) * (H + 2) * (W + 2) * 4
            A, Wt, out, keep = (heap(big) for _ in range(4))
            D.launches(lib)
            before = D.last_bounds(lib)[0]
            rc = lib.ard_conv_fwd_blocks(D.BF16, N, Cc, H, W, Cout, k, k, stride, pad, x, y, A, Wt, keep, out, ws, n, None)
            assert rc == 0, lib.ard_last_error().decode()
            names = D.launches(lib)[1]
            assert ("gemm_direct_kernel" in names) == fast, (N, Cc, Cout, x, y, names)
            assert ("conv_gemm_kernel" in names) == (not fast)
            if fast:   # the plan rides in the copy's launch
                assert "block_plan_kernel" not in names and "to_grid_src_kernel" in names, (H, W, names)
            if fast:
                nb, six = D.last_bounds(lib)
                assert nb == 1 and 0 <= six[0] < six[1] <= six[2] and 0 <= six[3] < six[4] <= six[5]


def test_block_pattern_random_shapes_pass_the_proof():
    """Seeded random layers under the block pattern (forward, both gradient modes): whatever path dispatch picks,
    every LDS-direct launch passes the exhaustive bounds proof and every request is accepted or refused cleanly."""
    import random
    rnd = random.Random(52)
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        fast = 0
        for _ in range(60):
            k = rnd.choice((1, 3, 3, 5))
            pad = rnd.choice((0, k // 2))
            H, W = rnd.randint(k + 4, 30), rnd.randint(k + 4, 30)
            N, Cc, Cout = rnd.randint(1, 6), rnd.choice((8, 40, 64, 100, 128, 192, 256)), rnd.choice((24, 65, 128, 130, 256, 300))
            Ho, Wo = H + 2 * pad - k + 1, W + 2 * pad - k + 1
            x = rnd.choice((rnd.randint(1, Ho * Wo), max(1, Ho * Wo // rnd.randint(1, 8))))
            y = rnd.choice((0, 64 * k * k, 128 * k * k, k * k * rnd.randint(1, 70), rnd.randint(1, Cc * k * k)))
            n = lib.ard_conv_workspace_bytes(D.BF16, N, Cc, H, W, Cout, k, k, 1, pad)
            ws = heap(n)
            big = N * max(Cc, Cout) * (H + 2 * pad + 2) * (W + 2 * pad + 2) * 4
            A, Wt, dY, out, keep = (heap(big) for _ in range(5))
            D.launches(lib)
            rc = lib.ard_conv_fwd_blocks(D.BF16, N, Cc, H, W, Cout, k, k, 1, pad, x, y, A, Wt, keep, out, ws, n, None)
            assert rc == 0, (N, Cc, Cout, H, W, k, pad, x, y, lib.ard_last_error().decode())
            fast += "gemm_direct_kernel" in D.launches(lib)[1]
            for mode in (2, 3):
                rc = lib.ard_conv_bwd_blocks(mode, D.BF16, N, Cc, H, W, Cout, k, k, 1, pad, x, y, A, Wt, dY, keep, out, ws, n, None)
                assert rc == 0, (mode, N, Cc, Cout, H, W, k, pad, x, y, lib.ard_last_error().decode())
        assert fast >= 3, "the random shapes never reached the path that skips dropped blocks"
        assert D.last_bounds(lib)[0] >= fast      # (reading them also resets the count for the next test)


def test_a_shortened_operand_is_rejected():
    """The proof is tight: with every operand pretended 8 elements shorter than it is, the dense 4096^3
    product (whose loaders read their operands to the last byte) must be refused, and nothing launched."""
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        D.last_bounds(lib)
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 4096, 4096, 4096, None, None, 0, ops=(0,)), "dense")
        n, six = D.last_bounds(lib)
        assert n == 1 and six[1] == six[2] and six[4] == six[5]      # both operands read up to their end
        D.launches(lib)
        lib.ard_debug_set_extent_slack(8)
        rc = D.layer_calls(lib, heap, D.BF16, 4096, 4096, 4096, None, None, 0, ops=(0,))
        assert rc == [-2] and "bounds proof" in lib.ard_last_error().decode()
        assert D.launches(lib)[0] == 0


def test_grouped_launch_of_a_dependency_level():
    """Independent calls recorded between ard_batch_begin and ard_batch_launch become one launch of the
    grouped kernel (plus one for their finishing passes); kernels the batch cannot hold are issued at once."""
    with D.dry_run() as lib:
        heap = D.FakeHeap()
        p1, p2 = (3, 2), (5, 1)
        assert lib.ard_batch_begin() == 0
        assert lib.ard_batch_begin() == -1            # already open
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 2048, p2, p1, IN | OUT | WC, ops=(1, 2)), "level 4")
        assert D.launches(lib)[0] == 0                # everything recorded
        assert lib.ard_batch_launch(None) == 0
        n, names = D.launches(lib)
        assert names[0] == "group_kernel" and n <= 2, names
        assert lib.ard_batch_launch(None) == -1       # no batch open
        # the three products of the 10-neuron layer: one launch
        lib.ard_batch_begin()
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 10, None, p2, IN | OUT), "level 3")
        assert lib.ard_batch_launch(None) == 0
        assert D.launches(lib) == (1, ["group_kernel"])
        # a call that gathers W itself issues the gather at once and records the product
        lib.ard_batch_begin()
        _ok(lib, D.layer_calls(lib, heap, D.BF16, 1024, 2048, 2048, p2, p1, IN | OUT, ops=(0,)), "gather inside")
        assert D.launches(lib) == (1, ["compact_weight_kernel"])
        assert lib.ard_batch_launch(None) == 0
        assert D.launches(lib) == (1, ["gemm_direct_kernel"])
        # fp32 is never recorded; abort drops a batch
        lib.ard_batch_begin()
        _ok(lib, D.layer_calls(lib, heap, D.F32, 64, 784, 1024, (2, 1), None, 0, ops=(0,)), "fp32")
        assert D.launches(lib)[0] >= 1
        lib.ard_batch_abort()
        assert lib.ard_batch_launch(None) == -1
