"""GPU parity of layers with at most 16 output neurons (the classifier layer, whose outputs are never
dropped): every layout the narrow-layer kernels take, against the oracle's masked-dense products."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from paper_2203_05705_amd import binding as ard
from util import assert_parity, from_vals, raw_bits, stored

pytestmark = pytest.mark.gpu

CASES = [  # B, I, O, pattern on the inputs (dp, b) or None
    (70, 136, 10, (3, 1)),
    (1000, 520, 10, (2, 2)),
    (129, 2048, 16, (4, 3)),
    (64, 264, 3, (5, 5)),
    (48, 96, 10, None),
    (33, 1030, 7, (2, 1)),
]


def compact_in(vals):
    return ard.pad_compact(from_vals(vals, "bf16"))


def check_compact(t, ref, what):
    n = ref.shape[1]
    assert t.shape == (ref.shape[0], ard.pad8(n)), (what, t.shape)
    assert_parity(t[:, :n].contiguous(), ref, "bf16", what=what)
    assert not t[:, n:].contiguous().view(torch.int16).any(), what + ": padding not +0.0"


@pytest.mark.parametrize("B,I,O,pi", CASES)
def test_narrow_layer_all_layouts(B, I, O, pi):
    print(f"narrow layer B={B} I={I} O={O} pat_in={pi}", flush=True)
    dtype = "bf16"
    rng = np.random.default_rng(B * 7 + I + O)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    srcv = stored(rng.standard_normal((B, I)), dtype)
    mo = np.ones(O, np.uint8)
    mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
    ki = P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    pat_i = ard.Pattern.row(*pi) if pi else None
    IN, OUT, WC, DW = ard.IN_COMPACT, ard.OUT_COMPACT, ard.W_COMPACT, ard.DW_COMPACT
    refY = G.drop_gemm_fwd(Xv, Wv, MW, mo, 1.25, relu=True)
    refdX = G.drop_gemm_bwd_data(dYv, Wv, MW, mo, -0.5) * (srcv > 0)
    refdW = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo)
    Xc, dYc, srcc = compact_in(Xv[:, ki]), compact_in(dYv), compact_in(srcv[:, ki])
    W, dY = from_vals(Wv, dtype), from_vals(dYv, dtype)
    Wc = ard.compact_weight(W, None, pat_i)

    # forward: compact activations in, dense W or its compact form, dense or compact Y
    for flags, Wt in ((IN, W), (IN | WC, Wc), (IN | OUT, W), (IN | OUT | WC, Wc)):
        Y = ard.drop_gemm_fwd(Xc, Wt, None, pat_i, alpha=1.25, relu=True, flags=flags, I=I, O=O)
        if flags & OUT:
            check_compact(Y, refY, f"Y flags={flags}")
        else:
            assert_parity(Y, refY, dtype, what=f"Y flags={flags}")

    # data gradient into the compact layout, with the mask of the layer below; negative alpha: padding stays +0.0
    for flags, Wt, dYt in ((IN, W, dY), (IN | WC, Wc, dY), (IN | OUT, W, dYc), (IN | OUT | WC, Wc, dYc)):
        dX = torch.full((B, ard.pad8(len(ki))), float("nan"), dtype=torch.bfloat16, device="cuda")
        ard.drop_gemm_bwd_data(dYt, Wt, None, pat_i, alpha=-0.5, relu_src=srcc, flags=flags, out=dX, I=I, O=O)
        n = len(ki)
        assert_parity(dX[:, :n].contiguous(), refdX[:, ki], dtype, what=f"dX flags={flags}")
        assert not raw_bits(dX[:, n:].contiguous()).any(), f"dX flags={flags}: padding not +0.0"
        dropped_by_mask = (srcv[:, ki] <= 0)
        assert not raw_bits(dX[:, :n].contiguous())[dropped_by_mask].any(), "masked entries are not +0.0"

    # weight gradient: full matrix with exact zeros at the dropped inputs, or the compact one
    for flags, dYt in ((IN, dY), (IN | OUT, dYc)):
        dW = torch.full((O, I), float("nan"), dtype=torch.bfloat16, device="cuda")
        ard.drop_gemm_bwd_weight(dYt, Xc, None, pat_i, flags=flags, out=dW, I=I, O=O)
        assert_parity(dW, refdW, dtype, zero_mask=(MW == 0), what=f"dW flags={flags}")
    dWc = torch.full((ard.pad8(O), ard.pad8(len(ki))), float("nan"), dtype=torch.bfloat16, device="cuda")
    ard.drop_gemm_bwd_weight(dYc, Xc, None, pat_i, flags=IN | OUT | DW, out=dWc, I=I, O=O)
    assert_parity(dWc[:O, :len(ki)].contiguous(), refdW[:, ki], dtype, what="dW compact")
    bits = raw_bits(dWc)
    assert not bits[O:, :].any() and not bits[:, len(ki):].any(), "dW compact: padding not +0.0"


def test_narrow_layer_dense_operands():
    """No pattern and no layout flag: dense X, W, dY with a width that allows 16-byte rows."""
    B, I, O, dtype = 200, 256, 10, "bf16"
    rng = np.random.default_rng(5)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    mo, mi = np.ones(O, np.uint8), np.ones(I, np.uint8)
    MW = G.weight_mask_rows(mo, mi)
    X, W, dY = (from_vals(v, dtype) for v in (Xv, Wv, dYv))
    assert_parity(ard.drop_gemm_fwd(X, W), G.drop_gemm_fwd(Xv, Wv, MW, mo, 1.0), dtype, what="Y")
    assert_parity(ard.drop_gemm_bwd_data(dY, W), G.drop_gemm_bwd_data(dYv, Wv, MW, mo, 1.0), dtype, what="dX")
    assert_parity(ard.drop_gemm_bwd_weight(dY, X), G.drop_gemm_bwd_weight(dYv, Xv, MW, mo), dtype, what="dW")
