#!/usr/bin/env python3
"""Benchmark of the Approximate Random Dropout hot path on one MI355X.

Headline workload (BASELINE config 2): MLP 784-2048-2048-10, batch 1024, bf16
inputs with fp32 accumulation, row-based dropout on both hidden layers, a new
pattern (dp, b) sampled per iteration and layer from the searched distribution.
One step = one training iteration: 3 forward GEMMs (ReLU fused), 3 weight-gradient
GEMMs and 2 data-gradient GEMMs (ReLU backward fused), all through libard's C ABI.

By default the calls of an iteration are issued one by one on one stream.  `--exec graph`
replays one captured HIP graph per iteration in which the weight gradients and weight
compactions run on a second lane beside the activation chain; on this machine the
cross-stream edges cost more than the overlap gains, so it is not the default.  The
vendor dense baseline (torch.matmul) is timed both ways and its better time is used.

Prints ONE JSON line.  `value` is the effective TFLOP/s (dense-equivalent FLOPs of
the iteration / time) at target rate 0.5 with inputs resident in HBM; the same
figures at rates 0.3 and 0.7, the speedups over the dense chain (this library at
dp=1 and the vendor GEMM through torch.matmul) and the other workloads' numbers
ride along under "rates" and "extra".
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_BF16 = 2500.0  # TFLOP/s, dense bf16 on MI355X
SIZES = (784, 2048, 2048, 10)
BATCH = 1024
N_PATTERNS = 8           # dp_max of the searched distribution
SEED = 2
# HBM bytes per launch of the dominant call's GEMM kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of `bench.py --exec eager` (summaries under profiles/); None until measured
TRAFFIC_BYTES = {"L2.bwd_weight": 16677504}   # 11366 KiB fetched + 4921 KiB written per launch


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--exec", dest="mode", choices=("eager", "graph"), default="eager",
                    help="eager: the calls are issued one by one on one stream (default, the faster one on this "
                         "machine); graph: every iteration is one replay of a captured two-lane HIP graph")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy 10 times (reference for the HBM traffic counters)")
    ap.add_argument("--only-call", default=None, metavar="NAME",
                    help="profiling aid: after one full warm-up pass, issue only this call of the rate-0.5 plans "
                         "(e.g. L2.bwd_weight) for --steps iterations, print its average time and exit")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (cpu_baseline) leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    return ap.parse_args()


class MlpChain:
    """Device buffers and prebuilt C-ABI argument lists for the config-2 iteration.

    An iteration is a small dependency graph, not a chain: the three weight gradients and the two
    weight compactions are leaves.  The plan puts them on a second lane (its own stream and
    workspace) so they overlap with the activation / data-gradient chain on the main lane."""

    def __init__(self, ard, torch, wl):
        to_dev = lambda a, _dt: ard.to_device(a)
        self.ard, self.torch = ard, torch
        self.lib = ard.lib()
        dt = torch.bfloat16
        self.X0 = to_dev(wl.arrays["X0"], "bf16")
        self.W = [to_dev(wl.arrays[f"W{l}"], "bf16") for l in (1, 2, 3)]
        self.dYL = to_dev(wl.arrays["dY"], "bf16")
        # the loss gradient in the compact layout (10 columns padded to 16, zero filled): 16-byte rows
        self.dYLc = ard.pad_compact(self.dYL)
        B = BATCH
        self.Y = [torch.empty((B, SIZES[l]), dtype=dt, device="cuda") for l in (1, 2, 3)]
        self.dYh = [torch.empty((B, SIZES[l]), dtype=dt, device="cuda") for l in (1, 2)]   # gradient at hidden outputs
        # room for the full [O x I] gradient and for the compact one, whose axes are padded to multiples of 8
        self.dW = [torch.empty(((w.shape[0] + 7) & ~7, (w.shape[1] + 7) & ~7), dtype=dt, device="cuda") for w in self.W]
        self.Wc = [torch.empty(((w.shape[0] + 7) & ~7, (w.shape[1] + 7) & ~7), dtype=dt, device="cuda")
                   for w in self.W[1:]]   # kept blocks of W2, W3 (axes padded to multiples of 8)
        self.ws = [torch.empty(1 << 24, dtype=torch.uint8, device="cuda") for _ in range(2)]  # one per lane
        self.main = torch.cuda.Stream()
        self.side = torch.cuda.Stream()
        self._keep = []

    def _pat(self, dp, b):
        p = self.ard.CPattern(self.ard.PAT_ROW, dp, b, 0, 0, 0, None, None, None, None, None)
        self._keep.append(p)
        return C.byref(p)

    def plan(self, pats, compact_dw=False):
        """pats = ((dp1,b1),(dp2,b2)) -> list of steps.

        A step is ("call", lane, fn, args, name, kept_flops) or ("wait", lane, other_lane): `lane`
        waits for everything issued so far on `other_lane`.  Lane 0 carries the forward chain and
        the data gradients, lane 1 the weight compactions and the weight gradients.  Issued on one
        stream in list order the plan is a valid sequential schedule too.

        Hidden activations and their gradients stay compact between the calls (only kept
        neurons are stored); W2's kept block is gathered once per iteration and shared by the
        forward and the data-gradient product (the 10-neuron last layer reads W3 through the map); weight gradients are written in full, or, with
        compact_dw, as the gradient of the kept synapses only (a reported variant, not the headline)."""
        lib, B = self.lib, BATCH
        p1, p2 = self._pat(*pats[0]), self._pat(*pats[1])
        k1 = -(-(SIZES[1] - (pats[0][1] - 1)) // pats[0][0])
        k2 = -(-(SIZES[2] - (pats[1][1] - 1)) // pats[1][0])
        X0, (W1, W2, W3), (Y1, Y2, Y3), (dY1, dY2), (dW1, dW2, dW3) = self.X0, self.W, self.Y, self.dYh, self.dW
        W2c, W3c = self.Wc
        dYL = self.dYLc
        bf = self.ard.BF16
        IN, OUT, WC = self.ard.IN_COMPACT, self.ard.OUT_COMPACT, self.ard.W_COMPACT
        DW1 = DW = 0
        if compact_dw:   # the compact gradients fit in the full-size buffers
            DW, DW1 = self.ard.DW_COMPACT, self.ard.DW_COMPACT | IN   # X0 has 784 = pad8(784) columns
        P = lambda t: t.data_ptr()
        f = 2.0 * B
        n = self.ws[0].numel()
        wsp = [P(w) for w in self.ws]
        st = [self.main.cuda_stream, self.side.cuda_stream]
        fwd, bwd_d, bwd_w, cw = lib.ard_drop_gemm_fwd, lib.ard_drop_gemm_bwd_data, lib.ard_drop_gemm_bwd_weight, lib.ard_compact_weight

        def call(lane, fn, args, name, flops):
            # the trailing arguments of every GEMM entry point are (workspace, bytes, stream)
            tail = (st[lane],) if fn is cw else (wsp[lane], n, st[lane])
            return ("call", lane, fn, args + tail, name, flops)
        # nothing dropped around layer 2 (the dense baseline, a (1, 1) sample): its products read W2 itself
        gather2 = pats[0][0] != 1 or pats[1][0] != 1
        W2x, WC2 = (W2c, WC) if gather2 else (W2, 0)
        return ([call(1, cw, (bf, SIZES[1], SIZES[2], P(W2), P(W2c), p2, p1), "L2.compact_w", 0.0)] if gather2 else []) + [
            call(0, fwd, (bf, B, SIZES[0], SIZES[1], P(X0), P(W1), P(Y1), p1, None, 1.0, 1, OUT), "L1.fwd", f * SIZES[0] * k1),
            ("wait", 0, 1),
            call(0, fwd, (bf, B, SIZES[1], SIZES[2], P(Y1), P(W2x), P(Y2), p2, p1, 1.0, 1, IN | OUT | WC2), "L2.fwd", f * k1 * k2),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[2], SIZES[3], P(dYL), P(Y2), P(dW3), None, p2, 1.0, 0.0, IN | OUT | DW), "L3.bwd_weight", f * k2 * SIZES[3]),
            call(0, fwd, (bf, B, SIZES[2], SIZES[3], P(Y2), P(W3), P(Y3), None, p2, 1.0, 0, IN), "L3.fwd", f * k2 * SIZES[3]),
            call(0, bwd_d, (bf, B, SIZES[2], SIZES[3], P(dYL), P(W3), P(dY2), None, p2, 1.0, P(Y2), IN | OUT), "L3.bwd_data", f * k2 * SIZES[3]),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[1], SIZES[2], P(dY2), P(Y1), P(dW2), p2, p1, 1.0, 0.0, IN | OUT | DW), "L2.bwd_weight", f * k1 * k2),
            call(0, bwd_d, (bf, B, SIZES[1], SIZES[2], P(dY2), P(W2x), P(dY1), p2, p1, 1.0, P(Y1), IN | OUT | WC2), "L2.bwd_data", f * k1 * k2),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[0], SIZES[1], P(dY1), P(X0), P(dW1), p1, None, 1.0, 0.0, OUT | DW1), "L1.bwd_weight", f * SIZES[0] * k1),
            ("wait", 0, 1),
        ]

    def calls(self, plan):
        return [s for s in plan if s[0] == "call"]

    def run(self, plan, lanes=2):
        """Issue one iteration.  lanes=1: everything on the main stream, waits are no-ops."""
        torch = self.torch
        streams = [self.main, self.side if lanes == 2 else self.main]
        for s in plan:
            if s[0] == "wait":
                if lanes == 2:
                    streams[s[1]].wait_stream(streams[s[2]])
                continue
            _, lane, fn, args, _, _ = s
            if lanes == 1 and lane == 1:
                args = args[:-1] + (self.main.cuda_stream,)
            rc = fn(*args)
            if rc != 0:
                raise RuntimeError(f"libard call {s[4]} failed with {rc}: {self.lib.ard_last_error().decode()}")

    def capture(self, plan):
        """One iteration as a HIP graph: lane 1 forks from and joins lane 0."""
        torch = self.torch
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=self.main):
            self.side.wait_stream(self.main)
            self.run(plan, lanes=2)
            self.main.wait_stream(self.side)
        return g

    def torch_dense_step(self, side=None):
        """The same iteration, dense, through the vendor GEMM (torch.matmul); weight gradients on
        the second lane when one is given."""
        t = self.torch
        main = t.cuda.current_stream()
        X0, (W1, W2, W3) = self.X0, self.W

        def on_side(fn):
            if side is None:
                return fn()
            side.wait_stream(main)
            with t.cuda.stream(side):
                return fn()
        Y1 = t.relu(X0 @ W1.t())
        Y2 = t.relu(Y1 @ W2.t())
        dW3 = on_side(lambda: self.dYL.t() @ Y2)
        Y3 = Y2 @ W3.t()
        dY2 = (self.dYL @ W3) * (Y2 > 0)
        dW2 = on_side(lambda: dY2.t() @ Y1)
        dY1 = (dY2 @ W2) * (Y1 > 0)
        dW1 = on_side(lambda: dY1.t() @ X0)
        if side is not None:
            main.wait_stream(side)
        return Y3, dW1, dW2, dW3


def dense_flops_per_iter():
    f = 2.0 * BATCH
    l1, l2, l3 = SIZES[0] * SIZES[1], SIZES[1] * SIZES[2], SIZES[2] * SIZES[3]
    return f * (2 * l1 + 3 * l2 + 3 * l3)      # fwd x3, dW x3, dX for L2 and L3


def spin_up(torch, seconds=0.3):
    """The GPU idles at a low clock: a short burst of dense work brings it to its running clock."""
    x = torch.randn((4096, 4096), device="cuda", dtype=torch.bfloat16)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            x @ x
        torch.cuda.synchronize()


def time_steps(torch, chain, plans, steps, warmup, mode):
    """Warm up, then time exactly `steps` iterations (plans are used round-robin).  Returns seconds."""
    n = len(plans)
    used = sorted({(warmup + it) % n for it in range(steps)} | {it % n for it in range(warmup)})
    with torch.cuda.stream(chain.main):
        if mode == "graph":
            graphs = {i: chain.capture(plans[i]) for i in used}   # capture costs are set-up, not step time
            step = lambda i: graphs[i].replay()
        else:
            step = lambda i: chain.run(plans[i], lanes=1)
        for it in range(warmup):
            step(it % n)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(steps):
            step((warmup + it) % n)
        torch.cuda.synchronize()
        return time.perf_counter() - t0


def time_torch_dense(torch, chain, steps, warmup, mode):
    with torch.cuda.stream(chain.main):
        if mode == "graph":
            chain.torch_dense_step(chain.side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=chain.main):
                keep = chain.torch_dense_step(chain.side)  # noqa: F841  (outputs live in the graph's pool)
            step = g.replay
        else:
            step = chain.torch_dense_step
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0


def per_call_times(torch, chain, plans, reps=3, only=None):
    """Per-call HIP-event durations (events on the stream the kernels run on), summed per call name
    over the plans; every call is issued once untimed and then `reps` times back to back inside its
    bracket.  `only`: issue just that call (one full iteration runs first so every buffer holds finite
    values; after that only the shapes of a plan matter for the time and the traffic of its calls)."""
    tot, cnt, flops = {}, {}, {}
    with torch.cuda.stream(chain.main):
        for i, plan in enumerate(plans):
            if only is None or i == 0:
                chain.run(plan, lanes=1)   # inputs of every call hold this plan's values (only: shapes suffice)
            for _, lane, fn, args, name, fl in chain.calls(plan):
                if only is not None and name != only:
                    continue
                if lane == 1:
                    args = args[:-1] + (chain.main.cuda_stream,)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                fn(*args)
                e0.record(chain.main)
                for _ in range(reps):
                    fn(*args)
                e1.record(chain.main)
                torch.cuda.synchronize()
                tot[name] = tot.get(name, 0.0) + e0.elapsed_time(e1) / reps
                cnt[name] = cnt.get(name, 0) + 1
                flops[name] = flops.get(name, 0.0) + fl
    return tot, cnt, flops


def cpu_baseline(wl, cdf, budget_s):
    """The oracle as it stands, timed on the host cores over a bounded number of iterations of the
    same workload (as many as fit in about `budget_s` seconds, at least 6)."""
    import numpy as np
    from oracle import gemm as G
    from oracle import patterns as P
    from oracle import rounding as R
    from oracle import sampler as S
    X0 = wl.values("X0")
    Ws = [wl.values(f"W{l}") for l in (1, 2, 3)]
    dYL = wl.values("dY")
    t0 = time.perf_counter()
    n_iter = 0
    while n_iter < 6 or (time.perf_counter() - t0 < budget_s and n_iter < 1000):
        pats = [S.sample_pattern(cdf, SEED, n_iter, layer) for layer in (1, 2)]
        masks = [P.row_mask(SIZES[l + 1], *pats[l]) for l in range(2)]
        G.mlp_iteration(X0, Ws, dYL, masks, R.to_bf16_values)
        n_iter += 1
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return dict(value=dense_flops_per_iter() * n_iter / dt / 1e12, unit="effective TFLOP/s", cores=threads,
                kind="oracle", sample=f"{n_iter} iterations of the config-2 MLP at target rate 0.5 (fp64 NumPy, masks materialised)",
                seconds=dt)


def extra_workloads(ard, torch):
    """Configs 3 (tile pattern, 4096^3 bf16, dp sweep and rate mixtures), 5 (convolution), 4 (LSTM), 1 and the
    HBM-bound passes: per-call times and speedups.  Short by design."""
    out = {}
    n = 4096
    g = torch.Generator(device="cuda").manual_seed(3)
    X = torch.randn((n, n), generator=g, device="cuda").to(torch.bfloat16)
    W = (0.02 * torch.randn((n, n), generator=g, device="cuda")).to(torch.bfloat16)
    dY = torch.randn((n, n), generator=g, device="cuda").to(torch.bfloat16)
    outb = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")

    def t_us(fn, reps=20, warm=5):
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3
    vendor = dict(fwd=t_us(lambda: torch.matmul(X, W.t(), out=outb)), bwd_data=t_us(lambda: torch.matmul(dY, W, out=outb)),
                  bwd_weight=t_us(lambda: torch.matmul(dY.t(), X, out=outb)))
    res = {"vendor_dense_us": vendor}
    ops = ("fwd", "bwd_data", "bwd_weight")
    for dp in range(1, N_PATTERNS + 1):
        pat = ard.Pattern.tile(dp, 1, 64, 64)
        pat = ard.Pattern.tile(dp, 1, 64, 64, lists=ard.pattern_gen(pat, n, n))
        kept = int(pat.lists["count"].item())
        flops = 2.0 * n * 64 * 64 * kept
        row = {}
        for name, fn in (("fwd", lambda: ard.drop_gemm_fwd(X, W, pat, out=outb, ws=ws)),
                         ("bwd_data", lambda: ard.drop_gemm_bwd_data(dY, W, pat, out=outb, ws=ws)),
                         ("bwd_weight", lambda: ard.drop_gemm_bwd_weight(dY, X, pat, out=outb, ws=ws))):
            us = t_us(fn)
            row[name] = dict(us=round(us, 1), kept_tflops=round(flops / us / 1e6, 1),
                             frac_mfma_peak=round(flops / us / 1e6 / MFMA_PEAK_BF16, 4))
        res[f"dp{dp}"] = row
    dense = {name: min(vendor[name], res["dp1"][name]["us"]) for name in ops}
    for name in ops:
        res["dp2"][name]["speedup_vs_dense"] = round(dense[name] / res["dp2"][name]["us"], 3)
    # target rates as mixtures over the searched distribution: expected time of the three products
    # under dp ~ K (per-dp times from the sweep above; the bias b only moves which tiles are kept)
    for p in (0.3, 0.5, 0.7):
        k, _ = ard.search_k(p, N_PATTERNS)
        t_mix = sum(float(k[dp - 1]) * sum(res[f"dp{dp}"][name]["us"] for name in ops) for dp in range(1, N_PATTERNS + 1))
        kept_frac = sum(float(k[dp - 1]) / dp for dp in range(1, N_PATTERNS + 1))
        res[f"rate{p}"] = dict(expected_us_fwd_bwd=round(t_mix, 1), speedup_vs_dense=round(sum(dense.values()) / t_mix, 3),
                               ideal_speedup=round(1.0 / kept_frac, 3))
    out["tile_gemm_4096_bf16_tile64"] = res
    out["conv_fmap_drop_128x256x28x28_bf16"] = extra_conv(ard, torch, t_us)
    out["lstm_1024_1024_b128_t64_bf16"] = extra_lstm(ard, torch, t_us)
    out["small_and_hbm_bound"] = extra_small(ard, torch, t_us)
    return out


def extra_small(ard, torch, t_us):
    """The latency- and HBM-bound pieces: config 1 (one fp32 layer, 64 x 784 -> 1024), pattern_gen, channel scoring."""
    from paper_2203_05705_amd import workloads as WL
    wl = WL.mlp_layer_f32()
    X, W, dY = (ard.to_device(wl.arrays[k]) for k in ("X", "W", "dY"))
    pat = ard.Pattern.row(2, 1)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
    Y, dX, dW = torch.empty((64, 1024), device="cuda"), torch.empty_like(X), torch.empty_like(W)
    res = {"config1_fp32_layer_us": dict(
        fwd=round(t_us(lambda: ard.drop_gemm_fwd(X, W, pat, out=Y, ws=ws)), 2),
        bwd_data=round(t_us(lambda: ard.drop_gemm_bwd_data(dY, W, pat, out=dX, ws=ws)), 2),
        bwd_weight=round(t_us(lambda: ard.drop_gemm_bwd_weight(dY, X, pat, out=dW, ws=ws)), 2))}
    tp = ard.Pattern.tile(3, 2, 64, 64)
    res["pattern_gen_us"] = dict(rows_2048=round(t_us(lambda: ard.pattern_gen(ard.Pattern.row(3, 2), 2048)), 2),
                                 tiles_64x64_grid=round(t_us(lambda: ard.pattern_gen(tp, 4096, 4096)), 2),
                                 note="includes the binding's output allocations; one workgroup, latency-bound")
    wlc = WL.conv_layer()
    A = ard.to_device(wlc.arrays["A"])
    N, C, H, Wd = A.shape
    wsc = torch.empty(ard.conv_workspace_bytes(ard.BF16, N, C, H, Wd, 256, 3, 3, 1, 1), dtype=torch.uint8, device="cuda")
    us = t_us(lambda: ard.conv_select(A, 0.5, ws=wsc))
    res["channel_score_select"] = dict(us=round(us, 1), bytes_read=A.numel() * 2,
                                       gb_per_s=round(A.numel() * 2 / us / 1e3, 1), frac_hbm_peak=round(A.numel() * 2 / us / 1e3 / 8000.0, 4))
    return res


def extra_conv(ard, torch, t_us):
    """Config 5: 3x3 convolution, N=128, C=Cout=256, 28x28, half of the input feature maps dropped."""
    import torch.nn.functional as F
    from paper_2203_05705_amd import workloads as WL
    wl = WL.conv_layer()
    A, Wt, dY = (ard.to_device(wl.arrays[k]) for k in ("A", "Wt", "dY"))
    N, C, H, W = A.shape
    ws = torch.empty(ard.conv_workspace_bytes(ard.BF16, N, C, H, W, 256, 3, 3, 1, 1), dtype=torch.uint8, device="cuda")
    res = {}
    for rate in (0.0, 0.5):
        sel = ard.conv_select(A, rate, ws=ws)
        nk = int(sel["count"].item())
        fl = 2.0 * N * H * W * 256 * nk * 9
        row = {"kept_channels": nk, "select_us": round(t_us(lambda: ard.conv_select(A, rate, ws=ws)), 1)}
        for name, fn in (("fwd", lambda: ard.conv_fwd(A, Wt, sel["keep"], nk, ws=ws)),
                         ("bwd_data", lambda: ard.conv_bwd_data(dY, Wt, sel["keep"], nk, (H, W), ws=ws)),
                         ("bwd_weight", lambda: ard.conv_bwd_weight(dY, A, sel["keep"], nk, ws=ws))):
            us = t_us(fn)
            row[name] = dict(us=round(us, 1), kept_tflops=round(fl / us / 1e6, 1), frac_mfma_peak=round(fl / us / 1e6 / MFMA_PEAK_BF16, 4))
        res[f"rate{rate}"] = row
    Ag, Wg = A.clone().requires_grad_(True), Wt.clone().requires_grad_(True)
    Y = F.conv2d(Ag, Wg, padding=1)
    res["vendor_dense_us"] = dict(fwd=round(t_us(lambda: F.conv2d(A, Wt, padding=1)), 1),
                                  bwd_data_plus_weight=round(t_us(lambda: torch.autograd.grad(Y, (Ag, Wg), dY, retain_graph=True)), 1))
    ours = sum(res["rate0.5"][k]["us"] for k in ("fwd", "bwd_data", "bwd_weight"))
    dense = min(sum(res["rate0.0"][k]["us"] for k in ("fwd", "bwd_data", "bwd_weight")),
                res["vendor_dense_us"]["fwd"] + res["vendor_dense_us"]["bwd_data_plus_weight"])
    res["speedup_vs_dense_rate0.5"] = round(dense / ours, 3)
    return res


def extra_lstm(ard, torch, t_us):
    """Config 4: LSTM layer, input 1024, hidden 1024, batch 128, 64 steps; row pattern on the hidden units."""
    from paper_2203_05705_amd import workloads as WL
    wl = WL.lstm_layer()
    x, Wl, dh = (ard.to_device(wl.arrays[k]) for k in ("x", "W", "dh"))
    T, B, I = x.shape
    Hh = Wl.shape[0] // 4
    res = {}
    for dp in (1, 2, 3):
        pat = ard.Pattern.row(dp, 1) if dp > 1 else None
        ws = torch.empty(ard.lstm_workspace_bytes(ard.BF16, T, B, I, Hh, pat), dtype=torch.uint8, device="cuda")
        h, c, g = ard.lstm_fwd(x, Wl, pat, ws=ws)
        res[f"dp{dp}"] = dict(fwd_us=round(t_us(lambda: ard.lstm_fwd(x, Wl, pat, ws=ws), reps=5, warm=2), 1),
                              bwd_us=round(t_us(lambda: ard.lstm_bwd(x, Wl, pat, h, c, g, dh, ws=ws), reps=5, warm=2), 1))
    lstm = torch.nn.LSTM(I, Hh).cuda().to(torch.bfloat16)
    xx = x.clone().requires_grad_(True)
    out_, _ = lstm(xx)
    res["vendor_dense_us"] = dict(fwd=round(t_us(lambda: lstm(xx), reps=5, warm=2), 1),
                                  bwd=round(t_us(lambda: torch.autograd.grad(out_, [xx] + list(lstm.parameters()), dh,
                                                                              retain_graph=True), reps=5, warm=2), 1))
    for dp in (1, 2, 3):
        res[f"dp{dp}"]["fwd_us_per_step"] = round(res[f"dp{dp}"]["fwd_us"] / T, 2)
    d = min(res["dp1"]["fwd_us"] + res["dp1"]["bwd_us"], res["vendor_dense_us"]["fwd"] + res["vendor_dense_us"]["bwd"])
    res["speedup_vs_dense_dp2"] = round(d / (res["dp2"]["fwd_us"] + res["dp2"]["bwd_us"]), 3)
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2203_05705_amd import binding as ard
    from paper_2203_05705_amd import workloads as WL
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (libard has no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    ard.lib()
    if args.copy_calibration:
        src = torch.ones(1 << 27, dtype=torch.int16, device="cuda")   # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 2, "copy_bytes_written": src.numel() * 2, "copies": 10}))
        return
    wl = WL.mlp_chain(seed=SEED, B=BATCH, sizes=SIZES)
    chain = MlpChain(ard, torch, wl)
    dense_f = dense_flops_per_iter()
    n_plan = max(100, args.steps + args.warmup)
    spin_up(torch)

    if args.only_call:
        _, cdf = ard.search_k(0.5, N_PATTERNS)
        pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(n_plan)]
        plans = [chain.plan(pp) for pp in pats]
        used = [plans[(args.warmup + it) % len(plans)] for it in range(args.steps)]
        tot, cnt, fl = per_call_times(torch, chain, used, only=args.only_call)
        name = args.only_call
        print(json.dumps({"call": name, "launches": cnt[name] * 4, "avg_us": tot[name] / cnt[name] * 1e3,
                          "kept_tflops": fl[name] / (tot[name] / 1e3) / 1e12}))
        return

    # dense chains: this library at dp=1, and the vendor GEMM, run the same way as the dropout chain
    dense_plan = [chain.plan(((1, 1), (1, 1)))]
    t_lib_dense = time_steps(torch, chain, dense_plan, args.steps, args.warmup, args.mode)
    t_vendor = {m: time_torch_dense(torch, chain, args.steps, args.warmup, m) for m in ("eager", "graph")}
    t_vendor_dense = min(t_vendor.values())
    t_dense = min(t_lib_dense, t_vendor_dense)

    rates, headline, roof = {}, None, None
    cdf05 = None
    for p in (0.3, 0.5, 0.7):
        _, cdf = ard.search_k(p, N_PATTERNS)
        if p == 0.5:
            cdf05 = cdf
        pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(n_plan)]
        plans = [chain.plan(pp) for pp in pats]
        dt = time_steps(torch, chain, plans, args.steps, args.warmup, args.mode)
        used = [plans[(args.warmup + it) % len(plans)] for it in range(args.steps)]
        kept_f = sum(c[5] for plan in used for c in chain.calls(plan))
        rates[str(p)] = dict(ms_per_step=dt / args.steps * 1e3, effective_tflops=dense_f * args.steps / dt / 1e12,
                             kept_tflops=kept_f / dt / 1e12, speedup_vs_lib_dense=t_lib_dense / dt,
                             speedup_vs_vendor_dense=t_vendor_dense / dt, speedup_vs_dense=t_dense / dt,
                             ideal_speedup=dense_f * args.steps / kept_f)
        if p == 0.5:
            headline = dt
            other = "eager" if args.mode == "graph" else "graph"
            rates[str(p)][f"{other}_ms_per_step"] = time_steps(torch, chain, plans, args.steps, args.warmup,
                                                               other) / args.steps * 1e3
            cplans = [chain.plan(pp, compact_dw=True) for pp in pats]
            rates[str(p)]["compact_dw_ms_per_step"] = time_steps(torch, chain, cplans, args.steps, args.warmup,
                                                                 args.mode) / args.steps * 1e3
            # roofline of the call that takes the largest share of the iteration, over the timed plans
            tot, cnt, fl = per_call_times(torch, chain, used)
            name = max(tot, key=tot.get)
            ksec = tot[name] / 1e3
            roof = dict(bound="mfma", kernel=f"gemm_direct_kernel ({name}; the call's finishing pass included)",
                        achieved=fl[name] / ksec / 1e12, peak=MFMA_PEAK_BF16, unit="TFLOP/s",
                        frac=fl[name] / ksec / 1e12 / MFMA_PEAK_BF16, avg_launch_us=ksec / cnt[name] * 1e6,
                        traffic=TRAFFIC_BYTES.get(name),
                        per_call_avg_us={k: round(v / cnt[k] * 1e3, 2) for k, v in tot.items()})
    dt = headline
    result = {
        "metric": "effective TFLOP/s + speedup vs dense GEMM at dropout 0.3/0.5/0.7, 1 MI355X",
        "value": dense_f * args.steps / dt / 1e12, "unit": "effective TFLOP/s (dense-equivalent FLOPs / time) at rate 0.5",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "MLP 784-2048-2048-10, batch 1024, bf16 in / fp32 accumulate, row-based dropout on both "
                               "hidden layers, pattern per iteration from the searched distribution (N=8); fwd + bwd",
                   "rate": 0.5, "seed": SEED,
                   "execution": "one HIP-graph replay per iteration, weight gradients on a second lane" if args.mode == "graph"
                                else "calls issued one by one on one stream"},
        "dense_ms_per_step": {"libard_dp1": t_lib_dense / args.steps * 1e3,
                              "vendor_torch_matmul_eager": t_vendor["eager"] / args.steps * 1e3,
                              "vendor_torch_matmul_graph": t_vendor["graph"] / args.steps * 1e3},
        "rates": rates, "roofline": roof,
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, cdf05, budget_s=12.0)
    if not args.no_extra:
        result["extra"] = extra_workloads(ard, torch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
