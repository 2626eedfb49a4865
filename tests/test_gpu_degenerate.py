"""GPU parity of the degenerate cases: patterns that keep nothing, and outputs that must then be all +0.0."""
import numpy as np
import pytest
import torch

from oracle import conv as OC
from oracle import gemm as G
from oracle import lstm as L
from oracle import rounding as R
from paper_2203_05705_amd import binding as ard
from util import assert_parity, from_vals, raw_bits, stored

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_list_pattern_that_keeps_no_output_neuron(dtype):
    """A row pattern always keeps a unit (dp <= number of units); an empty kept list keeps none."""
    B, I, O = 9, 16, 5
    rng = np.random.default_rng(3)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    mo = np.zeros(O, np.uint8)
    MW = G.weight_mask_rows(mo, np.ones(I, np.uint8))
    X, W, dY = (from_vals(v, dtype) for v in (Xv, Wv, dYv))
    pat = ard.Pattern.list(torch.empty(0, dtype=torch.int32, device="cuda"))
    for got, ref, what in ((ard.drop_gemm_fwd(X, W, pat), G.drop_gemm_fwd(Xv, Wv, MW, mo), "Y"),
                           (ard.drop_gemm_bwd_data(dY, W, pat), G.drop_gemm_bwd_data(dYv, Wv, MW, mo), "dX"),
                           (ard.drop_gemm_bwd_weight(dY, X, pat), G.drop_gemm_bwd_weight(dYv, Xv, MW, mo), "dW")):
        assert not np.any(ref), what
        assert not np.any(raw_bits(got)), what + " is not all +0.0"
    torch.cuda.synchronize()


def test_lstm_with_no_kept_unit():
    dtype, T, B, I, H = "bf16", 3, 4, 8, 6
    rng = np.random.default_rng(5)
    x = stored(rng.standard_normal((T, B, I)), dtype)
    W = stored(rng.uniform(-0.3, 0.3, (4 * H, I + H)), dtype)
    dh = stored(rng.standard_normal((T, B, H)), dtype)
    m = np.zeros(H, np.uint8)
    pat = ard.Pattern.list(torch.empty(0, dtype=torch.int32, device="cuda"))
    xd, Wd, dhd = (from_vals(v, dtype) for v in (x, W, dh))
    h, c, gates = ard.lstm_fwd(xd, Wd, pat)
    dx, dW = ard.lstm_bwd(xd, Wd, pat, h, c, gates, dhd)
    torch.cuda.synchronize()
    fwd = L.lstm_forward(x, W, m, R.to_bf16_values)
    bwd = L.lstm_backward(x, W, m, fwd, dh, R.to_bf16_values)
    assert not np.any(fwd["h"]) and not np.any(bwd["dx"]) and not np.any(bwd["dW"])
    for t, what in ((h, "h"), (c, "c"), (gates, "gates"), (dx, "dx"), (dW, "dW")):
        assert not np.any(raw_bits(t)), what + " is not all +0.0"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_conv_with_every_input_map_dropped(dtype):
    N, C, Cout, H, W = 2, 8, 16, 8, 8
    rng = np.random.default_rng(7)
    Av = stored(np.maximum(rng.standard_normal((N, C, H, W)), 0), dtype)
    Wv = stored(rng.standard_normal((Cout, C, 3, 3)) * 0.2, dtype)
    dYv = stored(rng.standard_normal((N, Cout, H, W)), dtype)
    Ad, Wd, dYd = (from_vals(v, dtype) for v in (Av, Wv, dYv))
    sel = ard.conv_select(Ad, 1.0)
    assert int(sel["count"].item()) == 0 and not sel["mask"].any()
    m = np.zeros(C, np.uint8)
    assert not np.any(OC.conv_fwd(Av, Wv, m))
    for t, what in ((ard.conv_fwd(Ad, Wd, sel["keep"], 0), "Y"), (ard.conv_bwd_data(dYd, Wd, sel["keep"], 0, (H, W)), "dA"),
                    (ard.conv_bwd_weight(dYd, Ad, sel["keep"], 0), "dW")):
        assert not np.any(raw_bits(t)), what + " is not all +0.0"
    torch.cuda.synchronize()
