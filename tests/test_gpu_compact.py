"""GPU parity of the compact-activation layout: a chain of layers keeps only the kept neurons
between calls; results must equal the oracle's masked-dense chain gathered on the kept units."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from oracle import patterns as P
from oracle import rounding as R
from paper_2203_05705_amd import binding as ard
from paper_2203_05705_amd import workloads as WL
from util import assert_parity, from_vals, stored, to_dev, to_host

pytestmark = pytest.mark.gpu


def compact_in(vals, dtype):
    """[B, count] values -> device tensor in the compact layout (pad8(count) columns, zero padded)."""
    return ard.pad_compact(from_vals(vals, dtype))


def check_compact(t, ref, dtype, what, rounded_ref=False):
    """Kept columns against the oracle; padding columns exactly +0.0."""
    n = ref.shape[1]
    assert t.shape == (ref.shape[0], ard.pad8(n)), (what, t.shape)
    assert_parity(t[:, :n].contiguous(), ref, dtype, what=what, rounded_ref=rounded_ref)
    assert not t[:, n:].contiguous().view(torch.int16 if dtype == "bf16" else torch.int32).any(), what + ": padding not +0.0"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,I,O,po,pi", [(70, 136, 90, (2, 2), (3, 1)), (130, 264, 200, (4, 2), (2, 2)),
                                          (64, 100, 83, (3, 3), None), (33, 96, 64, None, (5, 2))])
def test_single_layer_compact_layouts(dtype, B, I, O, po, pi):
    print(f"compact layer dtype={dtype} B={B} I={I} O={O} pat_out={po} pat_in={pi}", flush=True)
    rng = np.random.default_rng(B + I + O)
    Xv, Wv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (O, I), (B, O)))
    mo = P.row_mask(O, *po) if po else np.ones(O, np.uint8)
    mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    pat_o = ard.Pattern.row(*po) if po else None
    pat_i = ard.Pattern.row(*pi) if pi else None
    Xc, dYc = compact_in(Xv[:, ki], dtype), compact_in(dYv[:, ko], dtype)
    W = from_vals(Wv, dtype)
    IN, OUT, WC = ard.IN_COMPACT, ard.OUT_COMPACT, ard.W_COMPACT
    refY = G.drop_gemm_fwd(Xv, Wv, MW, mo, 1.5, relu=True)
    refdX = G.drop_gemm_bwd_data(dYv, Wv, MW, mo, 0.5)
    refdW = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo)
    # weight gathered inside the call
    Y = ard.drop_gemm_fwd(Xc, W, pat_o, pat_i, alpha=1.5, relu=True, flags=IN | OUT)
    check_compact(Y, refY[:, ko], dtype, "Y compact")
    dX = ard.drop_gemm_bwd_data(dYc, W, pat_o, pat_i, alpha=0.5, flags=IN | OUT)
    check_compact(dX, refdX[:, ki], dtype, "dX compact")
    # weight compacted once and shared
    Wc = ard.compact_weight(W, pat_o, pat_i)
    Wc_ref = np.zeros((ard.pad8(len(ko)), ard.pad8(len(ki))))
    Wc_ref[:len(ko), :len(ki)] = Wv[np.ix_(ko, ki)]
    assert np.array_equal(to_host(Wc), Wc_ref)
    Y2 = ard.drop_gemm_fwd(Xc, Wc, pat_o, pat_i, alpha=1.5, relu=True, flags=IN | OUT | WC, I=I, O=O)
    assert torch.equal(Y2, Y)
    dX2 = ard.drop_gemm_bwd_data(dYc, Wc, pat_o, pat_i, alpha=0.5, flags=IN | OUT | WC, I=I, O=O)
    assert torch.equal(dX2, dX)
    # mixed: compact in, expanded out (zero-filled)
    Y3 = ard.drop_gemm_fwd(Xc, W, pat_o, pat_i, alpha=1.5, relu=True, flags=IN)
    assert_parity(Y3, refY, dtype, zero_mask=(mo == 0)[None, :], what="Y expanded")
    # weight gradient: compact activations in, full matrix out
    dW = torch.full((O, I), float("nan"), dtype=W.dtype, device="cuda")
    ard.drop_gemm_bwd_weight(dYc, Xc, pat_o, pat_i, flags=IN | OUT, out=dW, I=I, O=O)
    assert_parity(dW, refdW, dtype, zero_mask=(MW == 0), what="dW")
    # weight gradient of the kept synapses only, in the layout of a compact weight
    dWc = torch.full((ard.pad8(len(ko)), ard.pad8(len(ki))), float("nan"), dtype=W.dtype, device="cuda")
    ard.drop_gemm_bwd_weight(dYc, Xc, pat_o, pat_i, flags=IN | OUT | ard.DW_COMPACT, out=dWc, I=I, O=O)
    check_compact_dw(dWc, refdW, ko, ki, dtype)
    with pytest.raises(ard.ArdError):
        ard.drop_gemm_bwd_weight(from_vals(dYv, dtype), Xc, pat_o, pat_i, flags=IN | ard.DW_COMPACT, I=I, O=O)


def check_compact_dw(dWc, refdW, ko, ki, dtype, rounded_ref=False):
    """Kept synapses against the oracle's full gradient; padding rows and columns exactly +0.0."""
    no, ni = len(ko), len(ki)
    assert dWc.shape == (ard.pad8(no), ard.pad8(ni))
    assert_parity(dWc[:no, :ni].contiguous(), refdW[np.ix_(ko, ki)], dtype, what="dW compact", rounded_ref=rounded_ref)
    bits = dWc.view(torch.int16 if dtype == "bf16" else torch.int32)
    assert not bits[no:, :].any() and not bits[:, ni:].any(), "dW compact: padding not +0.0"


@pytest.mark.parametrize("O,I,po,pi", [(2048, 2048, (2, 1), (2, 2)), (1000, 1500, (3, 2), (3, 1))])
def test_compact_weight_gradient_large(O, I, po, pi):
    """Compact weight gradient at sizes that run the split contraction over several macro tiles."""
    B, dtype = 128, "bf16"
    print(f"compact dW B={B} I={I} O={O} pat_out={po} pat_in={pi}", flush=True)
    rng = np.random.default_rng(O + I)
    Xv, dYv = (stored(rng.standard_normal(s), dtype) for s in ((B, I), (B, O)))
    mo, mi = P.row_mask(O, *po), P.row_mask(I, *pi)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    refdW = G.drop_gemm_bwd_weight(dYv, Xv, G.weight_mask_rows(mo, mi), mo)
    dWc = ard.drop_gemm_bwd_weight(compact_in(dYv[:, ko], dtype), compact_in(Xv[:, ki], dtype), ard.Pattern.row(*po),
                                   ard.Pattern.row(*pi), flags=ard.IN_COMPACT | ard.OUT_COMPACT | ard.DW_COMPACT, I=I, O=O)
    check_compact_dw(dWc, refdW, ko, ki, dtype)


@pytest.mark.parametrize("I", [1024, 1030])
def test_expanded_outputs_from_compact_inputs_large(I):
    """Compact operands in, full-size outputs out, at sizes where the product stores its scattered
    tile and the zeros of the dropped positions itself (16-byte rows for I = 1024, odd tail for 1030)."""
    B, O, po, pi, dtype = 1024, 768, (2, 1), (3, 2), "bf16"
    print(f"expanded outputs B={B} I={I} O={O} pat_out={po} pat_in={pi}", flush=True)
    rng = np.random.default_rng(I)
    Xv, Wv, dYv = (stored(rng.standard_normal(s) * sc, dtype) for s, sc in (((B, I), 1.0), ((O, I), 0.1), ((B, O), 1.0)))
    srcv = stored(rng.standard_normal((B, I)), dtype)
    mo, mi = P.row_mask(O, *po), P.row_mask(I, *pi)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    pat_o, pat_i = ard.Pattern.row(*po), ard.Pattern.row(*pi)
    Xc, dYc = compact_in(Xv[:, ki], dtype), compact_in(dYv[:, ko], dtype)
    W, src = from_vals(Wv, dtype), from_vals(srcv, dtype)
    Y = torch.full((B, O), float("nan"), dtype=W.dtype, device="cuda")
    ard.drop_gemm_fwd(Xc, W, pat_o, pat_i, alpha=0.5, relu=True, flags=ard.IN_COMPACT, out=Y)
    assert_parity(Y, G.drop_gemm_fwd(Xv, Wv, MW, mo, 0.5, relu=True), dtype, zero_mask=(mo == 0)[None, :], what="Y")
    dX = torch.full((B, I), float("nan"), dtype=W.dtype, device="cuda")
    ard.drop_gemm_bwd_data(dYc, W, pat_o, pat_i, relu_src=src, flags=ard.OUT_COMPACT, out=dX)
    ref = G.relu_bwd(G.drop_gemm_bwd_data(dYv, Wv, MW, mo, 1.0), srcv)
    assert_parity(dX, ref, dtype, zero_mask=(mi == 0)[None, :], what="dX")
    dW = torch.full((O, I), float("nan"), dtype=W.dtype, device="cuda")
    ard.drop_gemm_bwd_weight(dYc, Xc, pat_o, pat_i, flags=ard.IN_COMPACT | ard.OUT_COMPACT, out=dW, I=I, O=O)
    assert_parity(dW, G.drop_gemm_bwd_weight(dYv, Xv, MW, mo), dtype, zero_mask=(MW == 0), what="dW")
    torch.cuda.synchronize()


class _Config2:
    """An MLP chain workload on the device, loaded once per session: BASELINE config 2 (MLP 784-2048-2048-10,
    batch 1024, bf16) by default, or the same recipe at other sizes (Table 1 of the paper, batch 128)."""
    _cache = {}

    @classmethod
    def get(cls, sizes=(784, 2048, 2048, 10), B=1024):
        key = (tuple(sizes), B)
        if key not in cls._cache:
            wl = WL.mlp_chain(seed=2, B=B, sizes=tuple(sizes))
            c = cls()
            c.sizes, c.B = wl.params["sizes"], wl.params["B"]
            c.X0v, c.dYLv = wl.values("X0"), wl.values("dY")
            c.Wv = [wl.values(f"W{l}") for l in (1, 2, 3)]
            c.X0, c.dYL = to_dev(wl.arrays["X0"], "bf16"), to_dev(wl.arrays["dY"], "bf16")
            c.W = [to_dev(wl.arrays[f"W{l}"], "bf16") for l in (1, 2, 3)]
            c.dYLc = ard.pad_compact(c.dYL)
            c.batch_ws = [torch.empty(1 << 27, dtype=torch.uint8, device="cuda") for _ in range(3)]
            cls._cache = {key: c}      # one workload at a time stays on the device
        return cls._cache[key]


def _check_config2_iteration(pats, what, sizes=(784, 2048, 2048, 10), B=1024):
    """Every product the benchmark's plan issues for the patterns `pats` = ((dp1,b1),(dp2,b2)), with the
    benchmark's layout flags, each fed with the oracle's stored activations so that it is checked on its
    own: L1.fwd, L2.compact_w, L2.fwd, L3.fwd, L3.bwd_weight, L3.bwd_data, L2.bwd_weight, L2.bwd_data,
    L1.bwd_weight; plus the compact-W3 and unpadded-dY variants of the last layer."""
    # the oracle's chain rounds every stored tensor to bf16 where the kernels store it: rounded references
    from functools import partial
    check_compact_r = partial(check_compact, rounded_ref=True)
    check_compact_dw_r = partial(check_compact_dw, rounded_ref=True)
    assert_parity_r = partial(assert_parity, rounded_ref=True)
    c = _Config2.get(sizes, B)
    sizes, W = c.sizes, c.W
    IN, OUT, WC = ard.IN_COMPACT, ard.OUT_COMPACT, ard.W_COMPACT
    masks = [P.row_mask(sizes[l + 1], *pats[l]) for l in range(2)]
    keep = [P.keep_list(m) for m in masks]
    ref = G.mlp_iteration(c.X0v, c.Wv, c.dYLv, masks, R.to_bf16_values)
    p1, p2 = ard.Pattern.row(*pats[0]), ard.Pattern.row(*pats[1])
    Y1o = compact_in(ref["Y"][0][:, keep[0]], "bf16")
    Y2o = compact_in(ref["Y"][1][:, keep[1]], "bf16")
    dY2o = compact_in(ref["dY"][1][:, keep[1]], "bf16")
    dY1o = compact_in(ref["dY"][0][:, keep[0]], "bf16")
    # forward
    Y1 = ard.drop_gemm_fwd(c.X0, W[0], p1, None, relu=True, flags=OUT)
    check_compact_r(Y1, ref["Y"][0][:, keep[0]], "bf16", what + " Y1")
    gather2 = pats[0][0] != 1 or pats[1][0] != 1      # the benchmark's dense chain reads W2 itself
    if gather2:
        W2x, WC2 = ard.compact_weight(W[1], p2, p1), WC
        Wc_ref = np.zeros((ard.pad8(len(keep[1])), ard.pad8(len(keep[0]))))
        Wc_ref[:len(keep[1]), :len(keep[0])] = c.Wv[1][np.ix_(keep[1], keep[0])]
        assert np.array_equal(to_host(W2x), Wc_ref), what + " W2 compact"
    else:
        W2x, WC2 = W[1], 0
    Y2 = ard.drop_gemm_fwd(Y1o, W2x, p2, p1, relu=True, flags=IN | OUT | WC2, I=sizes[1], O=sizes[2])
    check_compact_r(Y2, ref["Y"][1][:, keep[1]], "bf16", what + " Y2")
    Y3 = ard.drop_gemm_fwd(Y2o, W[2], None, p2, flags=IN, I=sizes[2], O=sizes[3])
    assert_parity_r(Y3, ref["Y"][2], "bf16", what=what + " Y3")
    # backward
    zw3 = np.broadcast_to((masks[1] == 0)[None, :], ref["dW"][2].shape)
    dW3 = ard.drop_gemm_bwd_weight(c.dYLc, Y2o, None, p2, flags=IN | OUT, I=sizes[2], O=sizes[3])
    assert_parity_r(dW3, ref["dW"][2], "bf16", zero_mask=zw3, what=what + " dW3")
    dY2 = ard.drop_gemm_bwd_data(c.dYLc, W[2], None, p2, relu_src=Y2o, flags=IN | OUT, I=sizes[2], O=sizes[3])
    check_compact_r(dY2, ref["dY"][1][:, keep[1]], "bf16", what + " dY2")
    dW2 = ard.drop_gemm_bwd_weight(dY2o, Y1o, p2, p1, flags=IN | OUT, I=sizes[1], O=sizes[2])
    assert_parity_r(dW2, ref["dW"][1], "bf16", zero_mask=(G.weight_mask_rows(masks[1], masks[0]) == 0), what=what + " dW2")
    dY1 = ard.drop_gemm_bwd_data(dY2o, W2x, p2, p1, relu_src=Y1o, flags=IN | OUT | WC2, I=sizes[1], O=sizes[2])
    check_compact_r(dY1, ref["dY"][0][:, keep[0]], "bf16", what + " dY1")
    dW1 = ard.drop_gemm_bwd_weight(dY1o, c.X0, p1, None, flags=OUT, I=sizes[0], O=sizes[1])
    zw1 = np.broadcast_to((masks[0] == 0)[:, None], ref["dW"][0].shape)
    assert_parity_r(dW1, ref["dW"][0], "bf16", zero_mask=zw1, what=what + " dW1")
    # the benchmark's compact-gradient variant of the three weight gradients
    DW = ard.DW_COMPACT
    dW2c = ard.drop_gemm_bwd_weight(dY2o, Y1o, p2, p1, flags=IN | OUT | DW, I=sizes[1], O=sizes[2])
    check_compact_dw_r(dW2c, ref["dW"][1], keep[1], keep[0], "bf16")
    dW1c = ard.drop_gemm_bwd_weight(dY1o, c.X0, p1, None, flags=IN | OUT | DW, I=sizes[0], O=sizes[1])
    check_compact_dw_r(dW1c, ref["dW"][0], keep[0], np.arange(sizes[0]), "bf16")
    # other ways of issuing the last layer: W3 compacted, loss gradient not padded
    W3c = ard.compact_weight(W[2], None, p2)
    Y3c = ard.drop_gemm_fwd(Y2o, W3c, None, p2, flags=IN | WC, I=sizes[2], O=sizes[3])
    assert_parity_r(Y3c, ref["Y"][2], "bf16", what=what + " Y3 (compact W3)")
    dW3u = ard.drop_gemm_bwd_weight(c.dYL, Y2o, None, p2, flags=IN, I=sizes[2], O=sizes[3])
    assert_parity_r(dW3u, ref["dW"][2], "bf16", zero_mask=zw3, what=what + " dW3 (unpadded dY)")
    dY2u = ard.drop_gemm_bwd_data(c.dYL, W3c, None, p2, relu_src=Y2o, flags=IN | WC, I=sizes[2], O=sizes[3])
    check_compact_r(dY2u, ref["dY"][1][:, keep[1]], "bf16", what + " dY2 (unpadded dY, compact W3)")
    dY2c = ard.drop_gemm_bwd_data(c.dYLc, W3c, None, p2, relu_src=Y2o, flags=IN | OUT | WC, I=sizes[2], O=sizes[3])
    check_compact_r(dY2c, ref["dY"][1][:, keep[1]], "bf16", what + " dY2 (compact W3)")
    # the benchmark issues the independent calls of a dependency level as ONE grouped launch: the results
    # must be bit-identical to the calls issued one by one (every call of a batch has its own workspace)
    ws = c.batch_ws
    with ard.batch():
        Y1b = ard.drop_gemm_fwd(c.X0, W[0], p1, None, relu=True, flags=OUT, ws=ws[0])
        W2b = ard.compact_weight(W[1], p2, p1) if gather2 else None
    assert torch.equal(Y1b, Y1), what + " grouped Y1"
    assert W2b is None or torch.equal(W2b, W2x), what + " grouped W2 compact"
    with ard.batch():
        Y3b = ard.drop_gemm_fwd(Y2o, W[2], None, p2, flags=IN, I=sizes[2], O=sizes[3], ws=ws[0])
        dW3b = ard.drop_gemm_bwd_weight(c.dYLc, Y2o, None, p2, flags=IN | OUT, I=sizes[2], O=sizes[3], ws=ws[1])
        dY2b = ard.drop_gemm_bwd_data(c.dYLc, W[2], None, p2, relu_src=Y2o, flags=IN | OUT, I=sizes[2], O=sizes[3], ws=ws[2])
    assert torch.equal(Y3b, Y3) and torch.equal(dW3b, dW3) and torch.equal(dY2b, dY2), what + " grouped layer 3"
    with ard.batch():
        dW2b = ard.drop_gemm_bwd_weight(dY2o, Y1o, p2, p1, flags=IN | OUT, I=sizes[1], O=sizes[2], ws=ws[0])
        dY1b = ard.drop_gemm_bwd_data(dY2o, W2x, p2, p1, relu_src=Y1o, flags=IN | OUT | WC2, I=sizes[1], O=sizes[2], ws=ws[1])
    assert torch.equal(dW2b, dW2) and torch.equal(dY1b, dY1), what + " grouped layer 2 gradients"
    # a batch of one call, and a batch around a call that gathers W itself, behave like plain calls
    with ard.batch():
        Y2b = ard.drop_gemm_fwd(Y1o, W[1], p2, p1, relu=True, flags=IN | OUT, I=sizes[1], O=sizes[2], ws=ws[0])
    assert torch.equal(Y2b, Y2), what + " grouped Y2 (W gathered inside the call)"


@pytest.mark.parametrize("rate", [0.3, 0.5, 0.7])
def test_config2_mlp_chain_iterations(rate):
    """BASELINE config 2 at its three rates: patterns of iterations 0..4 from the searched distribution
    (Sections 3.3, 3.4), every product of the benchmark's plan against the oracle chain."""
    from oracle import sampler as S
    from oracle import search as K
    d, _ = K.search_k(rate, 8)
    cdf = [int(c) for c in K.fixed_point_cdf(d)]
    for it in range(5):
        pats = [S.sample_pattern(cdf, 2, it, layer) for layer in (1, 2)]
        assert pats == [ard.pattern_sample(cdf, 2, it, layer) for layer in (1, 2)]
        print(f"rate {rate} iteration {it}: patterns {pats}", flush=True)
        _check_config2_iteration(pats, f"rate {rate} it {it}")
    torch.cuda.synchronize()


@pytest.mark.parametrize("dp1", range(1, 9))
def test_config2_every_pattern_pair(dp1):
    """All 64 (dp1, dp2) period pairs the distribution with N = 8 can draw, one seeded bias each: the
    dispatch picks tile, split count and store path per (row step, column step, tile count), so every
    pair is its own launch configuration at the benchmark's size."""
    rng = np.random.default_rng(640 + dp1)
    for dp2 in range(1, 9):
        pats = [(dp1, int(rng.integers(1, dp1 + 1))), (dp2, int(rng.integers(1, dp2 + 1)))]
        print(f"pair {pats}", flush=True)
        _check_config2_iteration(pats, f"pair {pats}")
    torch.cuda.synchronize()


@pytest.mark.parametrize("h1,h2", [(1024, 64), (1024, 1024), (2048, 2048), (4096, 4096)])
def test_table1_networks_row_pattern(h1, h2):
    """The four hidden-layer shapes of the paper's Table 1 (Section 7.2.2), batch 128 (Section 7.2.1), rate 0.7:
    patterns of iterations 0..2 from the searched distribution, every product of the chain against the oracle."""
    from oracle import sampler as S
    from oracle import search as K
    d, _ = K.search_k(0.7, 8)
    cdf = [int(c) for c in K.fixed_point_cdf(d)]
    for it in range(3):
        pats = [S.sample_pattern(cdf, 2, it, layer) for layer in (1, 2)]
        print(f"table 1 network {h1}x{h2} iteration {it}: patterns {pats}", flush=True)
        _check_config2_iteration(pats, f"{h1}x{h2} it {it}", sizes=(784, h1, h2, 10), B=128)
    torch.cuda.synchronize()


@pytest.mark.parametrize("h1,h2,B", [(1024, 64, 128), (2048, 2048, 128), (4096, 4096, 128), (2048, 2048, 1024)])
def test_mlp_chain_under_tile_patterns(h1, h2, B):
    """Tile-based pattern (Section 3.2, 32 x 32 tiles as in the paper) on both hidden layers' weights: forward,
    data gradients with the ReLU backward fused, weight gradients, against the oracle's synapse-masked chain."""
    from oracle import sampler as S
    from oracle import search as K
    sizes = (784, h1, h2, 10)
    c = _Config2.get(sizes, B)
    d, _ = K.search_k(0.7, 8)
    cdf = [int(v) for v in K.fixed_point_cdf(d)]
    x = y = 32
    for it in range(2):
        pats = [S.sample_pattern(cdf, 2, it, layer) for layer in (1, 2)]
        print(f"tile chain {h1}x{h2} B={B} iteration {it}: patterns {pats}", flush=True)
        MWs = [P.expand_tile_mask(P.tile_mask(sizes[l + 1], sizes[l], x, y, *pats[l]), sizes[l + 1], sizes[l], x, y).astype(np.float64)
               for l in range(2)] + [np.ones((sizes[3], sizes[2]))]
        ref = G.mlp_iteration_masked(c.X0v, c.Wv, c.dYLv, MWs, R.to_bf16_values)
        t1, t2 = ard.Pattern.tile(*pats[0], x, y), ard.Pattern.tile(*pats[1], x, y)
        ap = lambda t, r, w, zm=None: assert_parity(t, r, "bf16", zero_mask=zm, what=f"tile chain it {it} {w}", rounded_ref=True)
        Y1o, Y2o = from_vals(ref["Y"][0], "bf16"), from_vals(ref["Y"][1], "bf16")
        dY2o, dY1o = from_vals(ref["dY"][1], "bf16"), from_vals(ref["dY"][0], "bf16")
        ap(ard.drop_gemm_fwd(c.X0, c.W[0], t1, relu=True), ref["Y"][0], "Y1")
        ap(ard.drop_gemm_fwd(Y1o, c.W[1], t2, relu=True), ref["Y"][1], "Y2")
        ap(ard.drop_gemm_fwd(Y2o, c.W[2]), ref["Y"][2], "Y3")
        ap(ard.drop_gemm_bwd_weight(c.dYL, Y2o), ref["dW"][2], "dW3")
        ap(ard.drop_gemm_bwd_data(c.dYL, c.W[2], relu_src=Y2o), ref["dY"][1], "dY2")
        ap(ard.drop_gemm_bwd_weight(dY2o, Y1o, t2), ref["dW"][1], "dW2", MWs[1] == 0)
        ap(ard.drop_gemm_bwd_data(dY2o, c.W[1], t2, relu_src=Y1o), ref["dY"][0], "dY1")
        ap(ard.drop_gemm_bwd_weight(dY1o, c.X0, t1), ref["dW"][0], "dW1", MWs[0] == 0)
    torch.cuda.synchronize()


@pytest.mark.parametrize("B,O,I,po,pi", [(256, 2044, 1024, (8, 3), (3, 2)), (8192, 520, 512, (8, 1), (2, 1)),
                                          (1024, 2048, 784, (8, 8), None)])
def test_weight_gradient_through_the_finishing_pass(B, O, I, po, pi):
    """Full-size dW from compact operands where the product leaves fp32 partial sums to a second pass:
    few kept rows (every 8th, row count not a multiple of 8), a contraction long enough to be split,
    and identity columns with 4 row tiles."""
    dtype = "bf16"
    print(f"finishing pass B={B} O={O} I={I} pat_out={po} pat_in={pi}", flush=True)
    rng = np.random.default_rng(B + O)
    Xv, dYv = (stored(rng.standard_normal(s) * 0.25, dtype) for s in ((B, I), (B, O)))
    mo = P.row_mask(O, *po)
    mi = P.row_mask(I, *pi) if pi else np.ones(I, np.uint8)
    ko, ki = P.keep_list(mo), P.keep_list(mi)
    MW = G.weight_mask_rows(mo, mi)
    refdW = G.drop_gemm_bwd_weight(dYv, Xv, MW, mo)
    dW = torch.full((O, I), float("nan"), dtype=torch.bfloat16, device="cuda")
    ard.drop_gemm_bwd_weight(compact_in(dYv[:, ko], dtype), compact_in(Xv[:, ki], dtype), ard.Pattern.row(*po),
                             ard.Pattern.row(*pi) if pi else None, flags=ard.IN_COMPACT | ard.OUT_COMPACT, out=dW, I=I, O=O)
    assert_parity(dW, refdW, dtype, zero_mask=(MW == 0), what="dW")
