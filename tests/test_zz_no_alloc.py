"""The weight gradient on the library's static scratch (the entry point for callers that cannot
allocate) against the workspace entry point: same kernels, so the outputs must be bit-identical; two
calls in a row, the second on a smaller layer; plus the oracle on both."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from paper_2203_05705_amd import binding as ard
from util import assert_parity, from_vals, raw_bits, stored

pytestmark = pytest.mark.gpu


def _case(B, O, I, po, pi, compact, seed):
    dtype = "bf16"
    rng = np.random.default_rng(seed)
    Xv, dYv = (stored(rng.standard_normal(s) * 0.25, dtype) for s in ((B, I), (B, O)))
    mo = P.row_mask(O, *po) if po else np.ones(O, np.uint8)
    mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    pat_o = ard.Pattern.row(*po) if po else None
    pat_i = ard.Pattern.row(*pi) if pi else None
    if compact:
        dY, X = ard.pad_compact(from_vals(dYv[:, ko], dtype)), ard.pad_compact(from_vals(Xv[:, ki], dtype))
        flags = ard.IN_COMPACT | ard.OUT_COMPACT
    else:
        dY, X, flags = from_vals(dYv, dtype), from_vals(Xv, dtype), 0
    ref = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo)
    return dY, X, pat_o, pat_i, flags, ref, MW


def test_static_scratch_weight_gradient_twice_in_a_row(guarded_outputs):
    lib = ard.lib()
    assert lib.ard_static_scratch_bytes() == 64 << 20
    # first: a contraction long enough to be split (fp32 partial sums + finishing pass in the scratch);
    # second, smaller: few kept rows scattered at element granularity (partial sums + finishing pass)
    cases = [(4096, 520, 512, (8, 1), (2, 1), True, 11), (256, 2044, 1024, (8, 3), (3, 2), True, 12),
             (300, 130, 72, (3, 2), None, False, 13)]
    for B, O, I, po, pi, compact, seed in cases:
        print(f"static scratch case B={B} O={O} I={I} pat_out={po} pat_in={pi} compact={compact}", flush=True)
        dY, X, pat_o, pat_i, flags, ref, MW = _case(B, O, I, po, pi, compact, seed)
        want = guarded_outputs.tensor((O, I), torch.bfloat16)
        ard.drop_gemm_bwd_weight(dY, X, pat_o, pat_i, flags=flags, out=want, I=I, O=O)
        got = guarded_outputs.tensor((O, I), torch.bfloat16)
        ard.drop_gemm_bwd_weight_static(dY, X, pat_o, pat_i, got, flags=flags, I=I, O=O)
        torch.cuda.synchronize()
        assert np.array_equal(raw_bits(got), raw_bits(want)), "static-scratch result differs from the workspace result"
        assert_parity(got, ref, "bf16", zero_mask=(MW == 0), what="dW (static scratch)")


def test_static_scratch_refuses_layers_beyond_its_size():
    lib = ard.lib()
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    rc = lib.ard_drop_gemm_bwd_weight_static(ard.BF16, 1024, 4096, 4096, t.data_ptr(), t.data_ptr(), t.data_ptr(), None, None,
                                             1.0, 0.0, 0, None)
    assert rc == -4 and b"static scratch" in lib.ard_last_error()
    torch.cuda.synchronize()
