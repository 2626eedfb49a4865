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
HBM_PEAK = 8000.0        # GB/s
SIZES = (784, 2048, 2048, 10)
BATCH = 1024
N_PATTERNS = 8           # dp_max of the searched distribution
SEED = 2
REPEATS = 5              # the block of `steps` timed iterations is repeated; median and min are reported
# HBM bytes per launch (fetched + written) of the kernels the roofline records describe.  A counter run
# cannot happen inside this program: the figures come from `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`
# runs of `bench.py --only-call NAME` (scaled by what the same counters read for a plain copy); the
# summaries, with their commands, are the files named here.  None: not measured.  L2.bwd_weight: per CALL, every
# kernel of the call (the product alone or grouped with the pass that zeroes dropped rows, the finishing pass
# where the pattern needs one), as its time is; the other two: the product kernel, per launch.
TRAFFIC = {
    "L2.bwd_weight": (20423402, "profiles/hbm_traffic_L2_bwd_weight.txt"),
    "C3.fwd.dp2": (151189085, "profiles/hbm_traffic_config3_fwd_dp2.txt"),
    "C5.fwd": (90894338, "profiles/hbm_traffic_config5_conv_fwd.txt"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--exec", dest="mode", choices=("grouped", "eager", "graph", "graph1"), default="grouped",
                    help="grouped (default): the independent calls of every dependency level of the iteration are "
                         "issued as one grouped launch (ard_batch_begin / ard_batch_launch), one stream; eager: the calls "
                         "are issued one by one on one stream; graph: every iteration is one replay of a captured "
                         "two-lane HIP graph of the eager calls; graph1: a single-lane HIP graph of the grouped launches")
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

    def __init__(self, ard, torch, wl, sizes=None, batch=None, ws_bytes=1 << 24):
        to_dev = lambda a, _dt: ard.to_device(a)
        self.ard, self.torch = ard, torch
        SIZES = self.sizes = tuple(sizes) if sizes else globals()["SIZES"]
        BATCH = self.B = batch if batch else globals()["BATCH"]
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
        p8 = ard.pad8
        self.dW = [torch.empty((p8(w.shape[0]), p8(w.shape[1])), dtype=dt, device="cuda") for w in self.W]
        self.Wc = [torch.empty((p8(w.shape[0]), p8(w.shape[1])), dtype=dt, device="cuda")
                   for w in self.W[1:]]   # kept blocks of W2, W3 (axes padded to multiples of 8)
        self.ws = [torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") for _ in range(3)]  # one per call of a level
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
        lib, B, SIZES = self.lib, self.B, self.sizes
        p1, p2 = self._pat(*pats[0]), self._pat(*pats[1])
        k1 = self.ard.kept_count(self.ard.Pattern.row(*pats[0]), SIZES[1])
        k2 = self.ard.kept_count(self.ard.Pattern.row(*pats[1]), SIZES[2])
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

        def call(lane, fn, args, name, flops, level, slot):
            # the trailing arguments of every GEMM entry point are (workspace, bytes, stream); `level` is the
            # call's depth in the iteration's dependency graph, `slot` its workspace within the level
            tail = (st[lane],) if fn is cw else (wsp[slot], n, st[lane])
            return ("call", lane, fn, args + tail, name, flops, level)
        # nothing dropped around layer 2 (the dense baseline, a (1, 1) sample): its products read W2 itself
        gather2 = pats[0][0] != 1 or pats[1][0] != 1
        W2x, WC2 = (W2c, WC) if gather2 else (W2, 0)
        return ([call(1, cw, (bf, SIZES[1], SIZES[2], P(W2), P(W2c), p2, p1), "L2.compact_w", 0.0, 0, 1)] if gather2 else []) + [
            call(0, fwd, (bf, B, SIZES[0], SIZES[1], P(X0), P(W1), P(Y1), p1, None, 1.0, 1, OUT), "L1.fwd", f * SIZES[0] * k1, 0, 0),
            ("wait", 0, 1),
            call(0, fwd, (bf, B, SIZES[1], SIZES[2], P(Y1), P(W2x), P(Y2), p2, p1, 1.0, 1, IN | OUT | WC2), "L2.fwd", f * k1 * k2, 1, 0),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[2], SIZES[3], P(dYL), P(Y2), P(dW3), None, p2, 1.0, 0.0, IN | OUT | DW), "L3.bwd_weight", f * k2 * SIZES[3], 2, 1),
            call(0, fwd, (bf, B, SIZES[2], SIZES[3], P(Y2), P(W3), P(Y3), None, p2, 1.0, 0, IN), "L3.fwd", f * k2 * SIZES[3], 2, 0),
            call(0, bwd_d, (bf, B, SIZES[2], SIZES[3], P(dYL), P(W3), P(dY2), None, p2, 1.0, P(Y2), IN | OUT), "L3.bwd_data", f * k2 * SIZES[3], 2, 2),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[1], SIZES[2], P(dY2), P(Y1), P(dW2), p2, p1, 1.0, 0.0, IN | OUT | DW), "L2.bwd_weight", f * k1 * k2, 3, 1),
            call(0, bwd_d, (bf, B, SIZES[1], SIZES[2], P(dY2), P(W2x), P(dY1), p2, p1, 1.0, P(Y1), IN | OUT | WC2), "L2.bwd_data", f * k1 * k2, 3, 0),
            ("wait", 1, 0),
            call(1, bwd_w, (bf, B, SIZES[0], SIZES[1], P(dY1), P(X0), P(dW1), p1, None, 1.0, 0.0, OUT | DW1), "L1.bwd_weight", f * SIZES[0] * k1, 4, 0),
            ("wait", 0, 1),
        ]

    def plan_tile(self, pats, tile=32):
        """The same iteration under TILE patterns (Section 3.2) on the two hidden layers' weights: synapses
        are dropped tile by tile, every neuron stays, so activations are full size and no weight is gathered."""
        lib, B, SIZES = self.lib, self.B, self.sizes
        A = self.ard
        mk = lambda dp, b: A.CPattern(A.PAT_TILE, dp, b, tile, tile, 0, None, None, None, None, None)
        t1, t2 = mk(*pats[0]), mk(*pats[1])
        self._keep += [t1, t2]
        t1, t2 = C.byref(t1), C.byref(t2)
        X0, (W1, W2, W3), (Y1, Y2, Y3), (dY1, dY2), (dW1, dW2, dW3) = self.X0, self.W, self.Y, self.dYh, self.dW
        P = lambda t: t.data_ptr()
        bf, n = A.BF16, self.ws[0].numel()
        wsp = [P(w) for w in self.ws]
        st = self.main.cuda_stream
        fwd, bwd_d, bwd_w = lib.ard_drop_gemm_fwd, lib.ard_drop_gemm_bwd_data, lib.ard_drop_gemm_bwd_weight
        f = 2.0 * B * tile * tile
        kt = lambda l, pat: -(-(-(-SIZES[l + 1] // tile) * -(-SIZES[l] // tile) - (pat[1] - 1)) // pat[0])   # kept tiles
        k1, k2 = kt(0, pats[0]), kt(1, pats[1])
        call = lambda fn, args, name, flops, level, slot: ("call", 0, fn, args + (wsp[slot], n, st), name, flops, level)
        return [
            call(fwd, (bf, B, SIZES[0], SIZES[1], P(X0), P(W1), P(Y1), t1, None, 1.0, 1, 0), "L1.fwd", f * k1, 0, 0),
            call(fwd, (bf, B, SIZES[1], SIZES[2], P(Y1), P(W2), P(Y2), t2, None, 1.0, 1, 0), "L2.fwd", f * k2, 1, 0),
            call(bwd_w, (bf, B, SIZES[2], SIZES[3], P(self.dYL), P(Y2), P(dW3), None, None, 1.0, 0.0, 0), "L3.bwd_weight", 2.0 * B * SIZES[2] * SIZES[3], 2, 1),
            call(fwd, (bf, B, SIZES[2], SIZES[3], P(Y2), P(W3), P(Y3), None, None, 1.0, 0, 0), "L3.fwd", 2.0 * B * SIZES[2] * SIZES[3], 2, 0),
            call(bwd_d, (bf, B, SIZES[2], SIZES[3], P(self.dYL), P(W3), P(dY2), None, None, 1.0, P(Y2), 0), "L3.bwd_data", 2.0 * B * SIZES[2] * SIZES[3], 2, 2),
            call(bwd_w, (bf, B, SIZES[1], SIZES[2], P(dY2), P(Y1), P(dW2), t2, None, 1.0, 0.0, 0), "L2.bwd_weight", f * k2, 3, 1),
            call(bwd_d, (bf, B, SIZES[1], SIZES[2], P(dY2), P(W2), P(dY1), t2, None, 1.0, P(Y1), 0), "L2.bwd_data", f * k2, 3, 0),
            call(bwd_w, (bf, B, SIZES[0], SIZES[1], P(dY1), P(X0), P(dW1), t1, None, 1.0, 0.0, 0), "L1.bwd_weight", f * k1, 4, 0),
        ]

    def calls(self, plan):
        return [s for s in plan if s[0] == "call"]

    def algorithmic_bytes(self, plan, name):
        """Bytes the named call of this plan has to move at least: its kept (compact) operands once and its
        result once -- a weight gradient written in full counts the whole [O x I] matrix, zeros included."""
        for s in self.calls(plan):
            if s[4] != name:
                continue
            _, B, I, O = s[3][:4]
            po, pi = s[3][7], s[3][8]
            k_of = lambda ref, units: units if ref is None else self.ard.kept_count(self.ard.Pattern.row(ref._obj.dp, ref._obj.b), units)
            Ok, Ik = k_of(po, O), k_of(pi, I)
            if name.endswith("bwd_weight"):
                return 2.0 * (B * Ok + B * Ik + O * I)
            return 2.0 * (B * Ik + Ok * Ik + B * Ok)
        return 0.0

    def run(self, plan, lanes=2):
        """Issue one iteration.  lanes=1: everything on the main stream, waits are no-ops."""
        torch = self.torch
        streams = [self.main, self.side if lanes == 2 else self.main]
        for s in plan:
            if s[0] == "wait":
                if lanes == 2:
                    streams[s[1]].wait_stream(streams[s[2]])
                continue
            _, lane, fn, args, _, _, _ = s
            if lanes == 1 and lane == 1:
                args = args[:-1] + (self.main.cuda_stream,)
            rc = fn(*args)
            if rc != 0:
                raise RuntimeError(f"libard call {s[4]} failed with {rc}: {self.lib.ard_last_error().decode()}")

    def run_grouped(self, plan):
        """Issue one iteration on the main stream, one grouped launch per dependency level: the calls of a
        level are independent of each other, each has its own workspace."""
        lib, stream = self.lib, self.main.cuda_stream
        calls = self.calls(plan)
        i = 0
        while i < len(calls):
            j = i
            while j < len(calls) and calls[j][6] == calls[i][6]:
                j += 1
            group = True   # (a single call may still be several kernels: zero fill + product)
            if group and lib.ard_batch_begin() != 0:
                raise RuntimeError(lib.ard_last_error().decode())
            for s in calls[i:j]:
                rc = s[2](*(s[3][:-1] + (stream,)))
                if rc != 0:
                    lib.ard_batch_abort()
                    raise RuntimeError(f"libard call {s[4]} failed with {rc}: {lib.ard_last_error().decode()}")
            if group and lib.ard_batch_launch(stream) != 0:
                raise RuntimeError(lib.ard_last_error().decode())
            i = j

    def capture_grouped(self, plan):
        """One iteration as a single-lane HIP graph of the grouped launches."""
        g = self.torch.cuda.CUDAGraph()
        with self.torch.cuda.graph(g, stream=self.main):
            self.run_grouped(plan)
        return g

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


def dense_flops_per_iter(sizes=None, batch=None):
    sizes, batch = sizes or SIZES, batch or BATCH
    f = 2.0 * batch
    l1, l2, l3 = sizes[0] * sizes[1], sizes[1] * sizes[2], sizes[2] * sizes[3]
    return f * (2 * l1 + 3 * l2 + 3 * l3)      # fwd x3, dW x3, dX for L2 and L3


def spin_up(torch, seconds=0.3):
    """The GPU idles at a low clock: a short burst of dense work brings it to its running clock."""
    x = torch.randn((4096, 4096), device="cuda", dtype=torch.bfloat16)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            x @ x
        torch.cuda.synchronize()


def _blocks(torch, step, n_steps, warmup, first_index=0):
    """Warm up, then time REPEATS blocks of exactly `n_steps` steps, each bracketed by a device
    synchronisation.  Returns the list of block times in seconds."""
    for it in range(warmup):
        step(first_index + it)
    out = []
    for r in range(REPEATS):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(n_steps):
            step(first_index + warmup + it)
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def _stat(blocks, n_steps):
    b = sorted(blocks)
    return dict(median=b[len(b) // 2] / n_steps, min=b[0] / n_steps, max=b[-1] / n_steps)


def time_steps(torch, chain, plans, steps, warmup, mode):
    """Times the iteration (plans are used round-robin; every repeat runs the same `steps` plans).
    Returns per-step seconds: dict(median, min, max)."""
    n = len(plans)
    used = sorted({(warmup + it) % n for it in range(steps)} | {it % n for it in range(warmup)})
    with torch.cuda.stream(chain.main):
        if mode == "graph":
            graphs = {i: chain.capture(plans[i]) for i in used}   # capture costs are set-up, not step time
            step = lambda i: graphs[i % n].replay()
        elif mode == "graph1":
            graphs = {i: chain.capture_grouped(plans[i]) for i in used}
            step = lambda i: graphs[i % n].replay()
        elif mode == "grouped":
            step = lambda i: chain.run_grouped(plans[i % n])
        else:
            step = lambda i: chain.run(plans[i % n], lanes=1)
        return _stat(_blocks(torch, step, steps, warmup), steps)


def time_torch_dense(torch, chain, steps, warmup, mode):
    with torch.cuda.stream(chain.main):
        if mode == "graph":
            chain.torch_dense_step(chain.side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=chain.main):
                keep = chain.torch_dense_step(chain.side)  # noqa: F841  (outputs live in the graph's pool)
            step = lambda i: g.replay()
        else:
            step = lambda i: chain.torch_dense_step()
        return _stat(_blocks(torch, step, steps, warmup), steps)


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
            for _, lane, fn, args, name, fl, _lvl in chain.calls(plan):
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


def per_level_times(torch, chain, plans, reps=3):
    """HIP-event time of each dependency level issued as a grouped launch (averaged over the plans; every
    level is issued once untimed and then `reps` times back to back inside its bracket)."""
    tot, cnt = {}, {}
    with torch.cuda.stream(chain.main):
        for plan in plans:
            chain.run_grouped(plan)
            calls = chain.calls(plan)
            for lvl in sorted({c[6] for c in calls}):
                sub = [c for c in calls if c[6] == lvl]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                chain.run_grouped(sub)
                e0.record(chain.main)
                for _ in range(reps):
                    chain.run_grouped(sub)
                e1.record(chain.main)
                torch.cuda.synchronize()
                key = "+".join(c[4] for c in sub)
                key = f"level{lvl}:" + ("+".join(c[4] for c in sub if c[4] != "L2.compact_w") + ("(+compact_w)" if any(c[4] == "L2.compact_w" for c in sub) else ""))
                tot[key] = tot.get(key, 0.0) + e0.elapsed_time(e1) / reps
                cnt[key] = cnt.get(key, 0) + 1
    return {k: round(v / cnt[k] * 1e3, 2) for k, v in sorted(tot.items())}, cnt


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
    # the same masked-dense products in fp32 (so that the CPU is not held back by the oracle's fp64): written
    # out here with NumPy, NOT the oracle and not checked against anything -- context for the figure above
    f32 = np.float32
    X0f, Wf, dYf = X0.astype(f32), [w.astype(f32) for w in Ws], dYL.astype(f32)
    t1 = time.perf_counter()
    n32 = 0
    while n32 < 6 or (time.perf_counter() - t1 < budget_s / 3 and n32 < 1000):
        pats = [S.sample_pattern(cdf, SEED, n32, layer) for layer in (1, 2)]
        m = [P.row_mask(SIZES[l + 1], *pats[l]).astype(f32) for l in range(2)]
        W1, W2, W3 = Wf[0] * m[0][:, None], Wf[1] * (m[1][:, None] * m[0][None, :]), Wf[2] * m[1][None, :]
        Y1 = np.maximum(X0f @ W1.T, 0)
        Y2 = np.maximum(Y1 @ W2.T, 0)
        Y3 = Y2 @ W3.T
        dW3 = (dYf.T @ Y2) * m[1][None, :]
        dY2 = (dYf @ W3) * (Y2 > 0)
        dW2 = (dY2.T @ Y1) * (m[1][:, None] * m[0][None, :])
        dY1 = (dY2 @ W2) * (Y1 > 0)
        dW1 = (dY1.T @ X0f) * m[0][:, None]
        n32 += 1
    dt32 = time.perf_counter() - t1
    return dict(value=dense_flops_per_iter() * n_iter / dt / 1e12, unit="effective TFLOP/s", cores=threads,
                kind="oracle", sample=f"{n_iter} iterations of the config-2 MLP at target rate 0.5 (fp64 NumPy, masks materialised)",
                seconds=dt,
                fp32_masked_dense=dict(value=dense_flops_per_iter() * n32 / dt32 / 1e12, unit="effective TFLOP/s", iterations=n32,
                                       seconds=dt32, note="same products in fp32 NumPy inside bench.py; not the oracle"))


def roofline_record(name, kernel, kept_flops, algo_bytes, launch_us, launches):
    """Both floors of one launch -- matrix cores (kept FLOPs / 2.5 PFLOP/s) and HBM (algorithmic bytes /
    8 TB/s) -- the binding one decides `bound`; `frac` is that floor over the measured launch time."""
    mfma_us = kept_flops / (MFMA_PEAK_BF16 * 1e12) * 1e6
    hbm_us = algo_bytes / (HBM_PEAK * 1e9) * 1e6
    traffic, src = TRAFFIC.get(name, (None, None))
    if hbm_us > mfma_us:
        rec = dict(bound="hbm", achieved=algo_bytes / launch_us / 1e3, peak=HBM_PEAK, unit="GB/s", frac=hbm_us / launch_us)
    else:
        rec = dict(bound="mfma", achieved=kept_flops / launch_us / 1e6, peak=MFMA_PEAK_BF16, unit="TFLOP/s", frac=mfma_us / launch_us)
    rec.update(kernel=kernel, call=name, avg_launch_us=launch_us, launches_timed=launches, kept_flops_per_launch=kept_flops,
               algorithmic_bytes_per_launch=algo_bytes, floors_us=dict(mfma=mfma_us, hbm=hbm_us),
               frac_of_mfma_peak=mfma_us / launch_us, frac_of_hbm_peak=hbm_us / launch_us,
               traffic=traffic, traffic_source=src,
               traffic_over_algorithmic=(traffic / algo_bytes if traffic else None))
    return rec


def event_us(torch, fn, reps=20, warm=5, blocks=REPEATS, flush=None):
    """HIP-event time of fn() on the current stream, in microseconds: median and min over `blocks` blocks of
    `reps` back-to-back calls.  flush: a large tensor rewritten before every call (cache-cold figure; the
    rewrite sits outside the event bracket, so reps is 1 per bracket then)."""
    for _ in range(warm):
        fn()
    out = []
    for _ in range(blocks):
        if flush is None:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / reps * 1e3)
        else:
            tot = 0.0
            for _ in range(reps):
                flush.add_(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                torch.cuda.synchronize()
                tot += e0.elapsed_time(e1)
            out.append(tot / reps * 1e3)
    out.sort()
    return dict(median=out[len(out) // 2], min=out[0])


class TileGemm:
    """Config 3: 4096^3 bf16, 64 x 64 weight tiles dropped per the tile pattern (seeded host inputs)."""

    def __init__(self, ard, torch):
        from paper_2203_05705_amd import workloads as WL
        wl = WL.tile_gemm(seed=3)
        self.ard, self.torch = ard, torch
        self.n = wl.params["B"]
        self.X, self.W, self.dY = (ard.to_device(wl.arrays[k]) for k in ("X", "W", "dY"))
        self.out = torch.empty((self.n, self.n), dtype=torch.bfloat16, device="cuda")
        self.ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")

    def kept_tiles(self, dp, b):
        t = (self.n // 64) ** 2
        return -(-(t - (b - 1)) // dp)

    def ops(self, dp, b):
        ard = self.ard
        pat = ard.Pattern.tile(dp, b, 64, 64)
        return (("fwd", lambda: ard.drop_gemm_fwd(self.X, self.W, pat, out=self.out, ws=self.ws)),
                ("bwd_data", lambda: ard.drop_gemm_bwd_data(self.dY, self.W, pat, out=self.out, ws=self.ws)),
                ("bwd_weight", lambda: ard.drop_gemm_bwd_weight(self.dY, self.X, pat, out=self.out, ws=self.ws)))


def extra_tile_gemm(ard, torch, rooflines):
    tg = TileGemm(ard, torch)
    n, X, W, dY, outb = tg.n, tg.X, tg.W, tg.dY, tg.out
    ops = ("fwd", "bwd_data", "bwd_weight")
    vendor = dict(fwd=event_us(torch, lambda: torch.matmul(X, W.t(), out=outb)),
                  bwd_data=event_us(torch, lambda: torch.matmul(dY, W, out=outb)),
                  bwd_weight=event_us(torch, lambda: torch.matmul(dY.t(), X, out=outb)))
    res = {"vendor_dense_us": {k: round(v["median"], 1) for k, v in vendor.items()}}
    for dp in range(1, N_PATTERNS + 1):
        flops = 2.0 * n * 64 * 64 * tg.kept_tiles(dp, 1)
        row = {}
        for name, fn in tg.ops(dp, 1):
            t = event_us(torch, fn)
            us = t["median"]
            row[name] = dict(us=round(us, 1), us_min=round(t["min"], 1), kept_tflops=round(flops / us / 1e6, 1),
                             frac_mfma_peak=round(flops / us / 1e6 / MFMA_PEAK_BF16, 4))
        res[f"dp{dp}"] = row
    dense = {name: min(vendor[name]["median"], res["dp1"][name]["us"]) for name in ops}
    for name in ops:
        res["dp2"][name]["speedup_vs_dense"] = round(dense[name] / res["dp2"][name]["us"], 3)
    # dominant large-shape kernel: the forward product at dp = 2 (rate 0.5).  Algorithmic bytes: the kept
    # tiles of W, the columns of X under a kept tile (dp = 2 over an even tile grid keeps every other tile
    # column: half of X), and all of Y.
    kept = tg.kept_tiles(2, 1)
    rooflines.append(roofline_record("C3.fwd.dp2", "gemm_direct_kernel<true, true, 256, 256, 8, 0> (config 3, tile pattern dp=2, forward)",
                                     2.0 * n * 64 * 64 * kept, 2.0 * (n * n / 2 + 64 * 64 * kept + n * n),
                                     res["dp2"]["fwd"]["us"], 20 * REPEATS))
    # target rates: the three products under (dp, b) ~ the searched distribution, 100 sampled patterns each
    dense_sum = sum(dense.values())
    for p in (0.3, 0.5, 0.7):
        k, cdf = ard.search_k(p, N_PATTERNS)
        pats = [ard.pattern_sample(cdf, 3, it, 0) for it in range(100)]
        fns = [fn for dp, b in pats for _, fn in tg.ops(dp, b)]

        def all_patterns():
            for fn in fns:
                fn()
        t = event_us(torch, all_patterns, reps=1, warm=1, blocks=3)
        kept_frac = sum(tg.kept_tiles(dp, b) for dp, b in pats) / (len(pats) * (n // 64) ** 2)
        res[f"rate{p}"] = dict(patterns=len(pats), us_per_pattern_fwd_bwd=round(t["median"] / len(pats), 1),
                               speedup_vs_dense=round(dense_sum * len(pats) / t["median"], 3),
                               kept_fraction=round(kept_frac, 4), ideal_speedup=round(1.0 / kept_frac, 3),
                               target_speedup=round(1.0 / (1.0 - p), 3))
    return res


def extra_small(ard, torch):
    """The latency- and HBM-bound pieces: config 1 (one fp32 layer, 64 x 784 -> 1024), pattern_gen, channel scoring."""
    from paper_2203_05705_amd import workloads as WL
    wl = WL.mlp_layer_f32()
    X, W, dY = (ard.to_device(wl.arrays[k]) for k in ("X", "W", "dY"))
    pat = ard.Pattern.row(2, 1)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
    flush = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda")
    Y, dX, dW = torch.empty((64, 1024), device="cuda"), torch.empty_like(X), torch.empty_like(W)
    calls = dict(fwd=lambda: ard.drop_gemm_fwd(X, W, pat, out=Y, ws=ws),
                 bwd_data=lambda: ard.drop_gemm_bwd_data(dY, W, pat, out=dX, ws=ws),
                 bwd_weight=lambda: ard.drop_gemm_bwd_weight(dY, X, pat, out=dW, ws=ws))
    res = {"config1_fp32_layer_us": {k: round(event_us(torch, f)["median"], 2) for k, f in calls.items()},
           "config1_fp32_layer_us_cache_cold": {k: round(event_us(torch, f, reps=10, blocks=3, flush=flush)["median"], 2)
                                                for k, f in calls.items()}}
    # pattern_gen at the C ABI, outputs allocated once (the binding's convenience wrapper allocates them per call)
    lib, st = ard.lib(), torch.cuda.current_stream().cuda_stream
    rp, tp = ard.Pattern.row(3, 2).c(), ard.Pattern.tile(3, 2, 64, 64).c()
    o_row, o_tile = ard.pattern_gen(ard.Pattern.row(3, 2), 2048), ard.pattern_gen(ard.Pattern.tile(3, 2, 64, 64), 4096, 4096)
    P = lambda t: t.data_ptr()
    res["pattern_gen_us"] = dict(
        rows_2048=round(event_us(torch, lambda: lib.ard_pattern_gen(C.byref(rp), 2048, 0, P(o_row["mask"]), P(o_row["keep"]),
                                                                    P(o_row["count"]), None, None, None, st))["median"], 2),
        tiles_64x64_grid=round(event_us(torch, lambda: lib.ard_pattern_gen(
            C.byref(tp), 4096, 4096, P(o_tile["mask"]), P(o_tile["keep"]), P(o_tile["count"]), P(o_tile["rowptr"]),
            P(o_tile["colptr"]), P(o_tile["csc_rows"]), st))["median"], 2),
        note="one workgroup (two launches for a tile grid), latency-bound; outputs preallocated")
    wlc = WL.conv_layer()
    A = ard.to_device(wlc.arrays["A"])
    N, Cc, H, Wd = A.shape
    wsc = torch.empty(ard.conv_workspace_bytes(ard.BF16, N, Cc, H, Wd, 256, 3, 3, 1, 1), dtype=torch.uint8, device="cuda")
    sel = ard.conv_select(A, 0.5, ws=wsc)
    us = event_us(torch, lambda: ard.conv_select(A, 0.5, ws=wsc, out=sel))["median"]
    res["channel_score_select"] = dict(us=round(us, 1), bytes_read=A.numel() * 2,
                                       gb_per_s=round(A.numel() * 2 / us / 1e3, 1), frac_hbm_peak=round(A.numel() * 2 / us / 1e3 / HBM_PEAK, 4))
    del flush
    return res


def extra_conv(ard, torch, rooflines):
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
        row = {"kept_channels": nk}
        # the layer's three passes on one workspace: the forward pass builds the channels-last grid of the
        # kept maps, the data gradient that of dY, the weight gradient takes both
        both = ard.CONV_REUSE_A | ard.CONV_REUSE_DY
        Yb = ard.conv_fwd(A, Wt, sel["keep"], nk, ws=ws)
        dAb = ard.conv_bwd_data(dY, Wt, sel["keep"], nk, (H, W), ws=ws)
        dWb = ard.conv_bwd_weight(dY, A, sel["keep"], nk, ws=ws)
        for name, fn in (("fwd", lambda: ard.conv_fwd(A, Wt, sel["keep"], nk, ws=ws, out=Yb)),
                         ("bwd_data", lambda: ard.conv_bwd_data(dY, Wt, sel["keep"], nk, (H, W), ws=ws, out=dAb)),
                         ("bwd_weight", lambda: ard.conv_bwd_weight(dY, A, sel["keep"], nk, ws=ws, out=dWb, reuse=both)),
                         ("bwd_weight_own_grids", lambda: ard.conv_bwd_weight(dY, A, sel["keep"], nk, ws=ws, out=dWb))):
            t = event_us(torch, fn)
            us = t["median"]
            row[name] = dict(us=round(us, 1), us_min=round(t["min"], 1), kept_tflops=round(fl / us / 1e6, 1),
                             frac_mfma_peak=round(fl / us / 1e6 / MFMA_PEAK_BF16, 4))
        res[f"rate{rate}"] = row
        if rate == 0.5:
            rooflines.append(roofline_record(
                "C5.fwd", "to_grid + gemm_direct_kernel<true, true, 256, *, 8, 1> (config 5, 128 of 256 input maps kept, forward call)",
                fl, 2.0 * (N * nk * H * W + 256 * nk * 9 + N * 256 * H * W), row["fwd"]["us"], 20 * REPEATS))
    # the paper's own mechanism on the same layer (Sections 5.1, 5.2.1): sensitivity of bands of 8 output
    # positions from 30 % sampled values against threshold 0.5 (t = 50 %), rows dropped with possibility 0.3
    # (sensitive) / 0.7 (insensitive), forward pass over the kept rows only
    x = 8
    rows, RB, CB = ard.sens_regions(A.shape, (3, 3), 1, 1, x, 0)
    pred = ard.sens_predict(A, (3, 3), 1, 1, x, 0, 300, 500, 0.5, 5, 0)
    rp = ard.sens_row_pattern(pred["sens"], rows, x, 0.3, 0.7, 5, 0)
    nkr = int(rp["count"].item())
    Yr = ard.conv_fwd_rows(A, Wt, rp, nkr, ws=ws)
    lib, P = ard.lib(), (lambda t: t.data_ptr())
    st = torch.cuda.current_stream().cuda_stream
    t_pred = event_us(torch, lambda: lib.ard_sens_predict(ard.BF16, N, C, H, W, 3, 3, 1, 1, x, 0, 300, 500, 0.5, 5, 0, P(A),
                                                          P(pred["count"]), P(pred["samples"]), P(pred["sens"]), st))["median"]
    t_pat = event_us(torch, lambda: lib.ard_sens_row_pattern(N, rows, x, P(pred["sens"]), 0.3, 0.7, 5, 0, P(rp["mask"]), P(rp["keep"]),
                                                             P(rp["count"]), st))["median"]
    t_fwd = event_us(torch, lambda: ard.conv_fwd_rows(A, Wt, rp, nkr, ws=ws, out=Yr))["median"]
    dense_fwd = res["rate0.0"]["fwd"]["us"]
    gr = ard.conv_bwd_rows(dY, A, Wt, rp, ws=ws)
    # (the weight gradient takes the grid of A the forward pass left and the masked grid of dY the data gradient left)
    t_rbwd = event_us(torch, lambda: ard.conv_bwd_rows(dY, A, Wt, rp, ws=ws, out=gr, reuse=ard.CONV_REUSE_A | ard.CONV_REUSE_DY),
                      reps=5, warm=2)["median"]
    res["row_sensitivity_pattern"] = dict(kept_rows=nkr, rows=N * rows, kept_fraction=round(nkr / (N * rows), 4),
                                          predict_us=round(t_pred, 1), row_pattern_us=round(t_pat, 1), fwd_rows_us=round(t_fwd, 1),
                                          fwd_speedup_vs_all_rows=round(dense_fwd / t_fwd, 3),
                                          fwd_speedup_with_prediction=round(dense_fwd / (t_fwd + t_pred + t_pat), 3),
                                          bwd_data_plus_weight_us=round(t_rbwd, 1),
                                          bwd_passes="the ordinary passes, dY's dropped positions zeroed while it is copied into its grid (no work skipped)")
    # the block-based pattern of Section 5.2.2 on the same layer: blocks of 112 output positions (four rows) by one
    # 64-channel group over all taps, balanced groups; the forward pass skips the dropped blocks, the gradients run
    # the ordinary passes once per column block on a dY whose positions in that block's dropped bands are zeroed
    x, by = 112, 576
    predb = ard.sens_predict(A, (3, 3), 1, 1, x, by, 300, 500, 0.5, 5, 0)
    bp = ard.sens_block_pattern(predb, 1, 0.3, 0.7, 5, 0)
    Ybl = ard.conv_fwd_blocks(A, Wt, bp["keep"], x, by, ws=ws)
    gb = ard.conv_bwd_blocks(dY, A, Wt, bp["keep"], x, by, ws=ws)
    t_predb = event_us(torch, lambda: lib.ard_sens_predict(ard.BF16, N, C, H, W, 3, 3, 1, 1, x, by, 300, 500, 0.5, 5, 0, P(A),
                                                           P(predb["count"]), P(predb["samples"]), P(predb["sens"]), st))["median"]
    t_bpat = event_us(torch, lambda: ard.sens_block_pattern(predb, 1, 0.3, 0.7, 5, 0), reps=5, warm=2)["median"]
    t_bfwd = event_us(torch, lambda: ard.conv_fwd_blocks(A, Wt, bp["keep"], x, by, ws=ws, out=Ybl), reps=5, warm=2)["median"]
    t_bbwd = event_us(torch, lambda: ard.conv_bwd_blocks(dY, A, Wt, bp["keep"], x, by, ws=ws, out=gb), reps=5, warm=2)["median"]
    res["block_sensitivity_pattern"] = dict(kept_fraction=round(float(bp["keep"].float().mean().item()), 4), predict_us=round(t_predb, 1),
                                            block_pattern_us=round(t_bpat, 1), fwd_blocks_us=round(t_bfwd, 1),
                                            fwd_speedup_vs_all_blocks=round(dense_fwd / t_bfwd, 3),
                                            fwd_speedup_with_prediction=round(dense_fwd / (t_bfwd + t_predb + t_bpat), 3),
                                            bwd_data_plus_weight_us=round(t_bbwd, 1), blocks="112 x 576",
                                            bwd_passes="one ordinary pass per column block, dY masked while it is copied into its grid (no work skipped)")
    Ag, Wg = A.clone().requires_grad_(True), Wt.clone().requires_grad_(True)
    Y = F.conv2d(Ag, Wg, padding=1)
    res["vendor_dense_us"] = dict(fwd=round(event_us(torch, lambda: F.conv2d(A, Wt, padding=1))["median"], 1),
                                  bwd_data_plus_weight=round(event_us(torch, lambda: torch.autograd.grad(Y, (Ag, Wg), dY, retain_graph=True))["median"], 1))
    ours = sum(res["rate0.5"][k]["us"] for k in ("fwd", "bwd_data", "bwd_weight"))
    dense = min(sum(res["rate0.0"][k]["us"] for k in ("fwd", "bwd_data", "bwd_weight")),
                res["vendor_dense_us"]["fwd"] + res["vendor_dense_us"]["bwd_data_plus_weight"])
    res["speedup_vs_dense_rate0.5"] = round(dense / ours, 3)
    del Ag, Wg, Y
    # the same three passes on other 3x3 layer shapes (seeded random tensors; planes of 14 x 14 and 7 x 7 positions
    # are not whole numbers of 16-byte pieces, 7 x 7 leaves few output positions per image)
    other = {}
    for (n_, c_, h_, co_) in ((128, 512, 14, 512), (128, 512, 7, 512), (64, 128, 56, 128)):
        g = torch.Generator(device="cuda").manual_seed(SEED)
        A2 = torch.randn(n_, c_, h_, h_, device="cuda", generator=g).to(torch.bfloat16)
        dY2 = torch.randn(n_, co_, h_, h_, device="cuda", generator=g).to(torch.bfloat16)
        W2 = (torch.randn(co_, c_, 3, 3, device="cuda", generator=g) * 0.05).to(torch.bfloat16)
        ws2 = torch.empty(ard.conv_workspace_bytes(ard.BF16, n_, c_, h_, h_, co_, 3, 3, 1, 1), dtype=torch.uint8, device="cuda")
        row = {}
        for rate in (0.0, 0.5):
            sel = ard.conv_select(A2, rate, ws=ws2)
            nk = int(sel["count"].item())
            Yo = ard.conv_fwd(A2, W2, sel["keep"], nk, ws=ws2)
            dAo = ard.conv_bwd_data(dY2, W2, sel["keep"], nk, (h_, h_), ws=ws2)
            dWo = ard.conv_bwd_weight(dY2, A2, sel["keep"], nk, ws=ws2)
            both = ard.CONV_REUSE_A | ard.CONV_REUSE_DY
            row[f"rate{rate}"] = {
                "fwd": round(event_us(torch, lambda: ard.conv_fwd(A2, W2, sel["keep"], nk, ws=ws2, out=Yo), reps=5, warm=2)["median"], 1),
                "bwd_data": round(event_us(torch, lambda: ard.conv_bwd_data(dY2, W2, sel["keep"], nk, (h_, h_), ws=ws2, out=dAo), reps=5, warm=2)["median"], 1),
                "bwd_weight": round(event_us(torch, lambda: ard.conv_bwd_weight(dY2, A2, sel["keep"], nk, ws=ws2, out=dWo, reuse=both), reps=5, warm=2)["median"], 1)}
        row["speedup_rate0.5"] = round(sum(row["rate0.0"].values()) / sum(row["rate0.5"].values()), 3)
        other[f"N{n_}_C{c_}_{h_}x{h_}_Cout{co_}_us"] = row
        del A2, dY2, W2, ws2
    res["other_layer_shapes"] = other
    return res


def extra_lstm(ard, torch):
    """Config 4: LSTM layer, input 1024, hidden 1024, batch 128, 64 steps; row pattern on the hidden units."""
    from paper_2203_05705_amd import workloads as WL
    wl = WL.lstm_layer()
    x, Wl, dh = (ard.to_device(wl.arrays[k]) for k in ("x", "W", "dh"))
    T, B, I = x.shape
    Hh = Wl.shape[0] // 4
    res = {}
    flush = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda")
    for dp in (1, 2, 3):
        pat = ard.Pattern.row(dp, 1) if dp > 1 else None
        ws = torch.empty(ard.lstm_workspace_bytes(ard.BF16, T, B, I, Hh, pat), dtype=torch.uint8, device="cuda")
        h, c, g = ard.lstm_fwd(x, Wl, pat, ws=ws)
        out = (h, c, g)
        fwd = event_us(torch, lambda: ard.lstm_fwd(x, Wl, pat, ws=ws, out=out), reps=5, warm=2)
        bwd = event_us(torch, lambda: ard.lstm_bwd(x, Wl, pat, h, c, g, dh, ws=ws), reps=5, warm=2)
        res[f"dp{dp}"] = dict(fwd_us=round(fwd["median"], 1), bwd_us=round(bwd["median"], 1), fwd_us_min=round(fwd["min"], 1),
                              fwd_us_per_step=round(fwd["median"] / T, 2))
        if dp == 2:
            cold = event_us(torch, lambda: ard.lstm_fwd(x, Wl, pat, ws=ws, out=out), reps=3, warm=1, blocks=3, flush=flush)
            res["dp2"]["fwd_us_cache_cold"] = round(cold["median"], 1)
    # the TILE variant (Section 7.2.3): 32 x 32 tiles of the fused weight dropped, every unit kept; the products
    # run dense on the masked weight, so this row shows what the masking costs, not a gain
    tpat = ard.Pattern.tile(2, 1, 32, 32)
    ws = torch.empty(ard.lstm_workspace_bytes(ard.BF16, T, B, I, Hh, tpat), dtype=torch.uint8, device="cuda")
    out = ard.lstm_fwd(x, Wl, tpat, ws=ws)
    fwd = event_us(torch, lambda: ard.lstm_fwd(x, Wl, tpat, ws=ws, out=out), reps=5, warm=2)
    bwd = event_us(torch, lambda: ard.lstm_bwd(x, Wl, tpat, out[0], out[1], out[2], dh, ws=ws), reps=5, warm=2)
    res["tile32_dp2_masked_dense"] = dict(fwd_us=round(fwd["median"], 1), bwd_us=round(bwd["median"], 1))
    del flush
    lstm = torch.nn.LSTM(I, Hh).cuda().to(torch.bfloat16)
    xx = x.clone().requires_grad_(True)
    out_, _ = lstm(xx)
    res["vendor_dense_us"] = dict(fwd=round(event_us(torch, lambda: lstm(xx), reps=5, warm=2, blocks=3)["median"], 1),
                                  bwd=round(event_us(torch, lambda: torch.autograd.grad(out_, [xx] + list(lstm.parameters()), dh,
                                                                                         retain_graph=True), reps=5, warm=2, blocks=3)["median"], 1))
    d = min(res["dp1"]["fwd_us"] + res["dp1"]["bwd_us"], res["vendor_dense_us"]["fwd"] + res["vendor_dense_us"]["bwd"])
    res["speedup_vs_dense_dp2"] = round(d / (res["dp2"]["fwd_us"] + res["dp2"]["bwd_us"]), 3)
    return res


def extra_table1(ard, torch):
    """The network sweep of the paper's Table 1 (Section 7.2.2): MLP 784-h1-h2-10, batch 128, rate 0.7, ROW and
    TILE (32 x 32) patterns from the searched distribution, against the same chain with nothing dropped."""
    from paper_2203_05705_amd import workloads as WL
    _, cdf = ard.search_k(0.7, N_PATTERNS)
    paper = {(1024, 64): (1.27, 1.19), (1024, 1024): (1.45, 1.41), (2048, 2048): (1.77, 1.60), (4096, 4096): (2.16, 1.95)}
    res = {}
    for (h1, h2), (p_row, p_tile) in paper.items():
        sizes = (784, h1, h2, 10)
        chain = MlpChain(ard, torch, WL.mlp_chain(seed=SEED, B=128, sizes=sizes), sizes=sizes, batch=128, ws_bytes=1 << 26)
        pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(100)]
        t_dense = time_steps(torch, chain, [chain.plan(((1, 1), (1, 1)))], 50, 5, "grouped")["median"]
        t_row = time_steps(torch, chain, [chain.plan(pp) for pp in pats], 50, 5, "grouped")["median"]
        t_tile = time_steps(torch, chain, [chain.plan_tile(pp) for pp in pats], 50, 5, "grouped")["median"]
        res[f"{h1}x{h2}"] = dict(dense_us=round(t_dense * 1e6, 1), row_us=round(t_row * 1e6, 1), tile_us=round(t_tile * 1e6, 1),
                                 row_speedup=round(t_dense / t_row, 3), tile_speedup=round(t_dense / t_tile, 3),
                                 paper_row_speedup_gtx1080ti=p_row, paper_tile_speedup_gtx1080ti=p_tile)
        del chain
    return res


def extra_lstm_batch_scaling(ard, torch):
    """Section 7.2.3: LSTM layer with 1500 hidden units, sequence length 35, batch 20 and 40; row pattern on the
    hidden units at dp = 2 and 3 against dp = 1."""
    from paper_2203_05705_amd import workloads as WL
    res = {}
    for B in (20, 40):
        wl = WL.lstm_layer(seed=4, T=35, B=B, I=1500, H=1500)
        x, Wl, dh = (ard.to_device(wl.arrays[k]) for k in ("x", "W", "dh"))
        T, _, I = x.shape
        row = {}
        for dp in (1, 2, 3):
            pat = ard.Pattern.row(dp, 1) if dp > 1 else None
            ws = torch.empty(ard.lstm_workspace_bytes(ard.BF16, T, B, I, 1500, pat), dtype=torch.uint8, device="cuda")
            out = ard.lstm_fwd(x, Wl, pat, ws=ws)
            h, c, g = out
            gout = ard.lstm_bwd(x, Wl, pat, h, c, g, dh, ws=ws)
            fwd = event_us(torch, lambda: ard.lstm_fwd(x, Wl, pat, ws=ws, out=out), reps=5, warm=2, blocks=3)["median"]
            bwd = event_us(torch, lambda: ard.lstm_bwd(x, Wl, pat, h, c, g, dh, ws=ws, out=gout), reps=5, warm=2, blocks=3)["median"]
            row[f"dp{dp}_fwd_bwd_us"] = round(fwd + bwd, 1)
        row["speedup_dp2"] = round(row["dp1_fwd_bwd_us"] / row["dp2_fwd_bwd_us"], 3)
        row["speedup_dp3"] = round(row["dp1_fwd_bwd_us"] / row["dp3_fwd_bwd_us"], 3)
        res[f"batch{B}"] = row
    return res


def only_call(args, ard, torch, chain):
    """Profiling aid: issue one call in a tight loop so that a rocprofv3 run sees little else."""
    name = args.only_call
    if name in ("C3.fwd.dp2", "C5.fwd"):
        if name == "C3.fwd.dp2":
            fn = dict(TileGemm(ard, torch).ops(2, 1))["fwd"]
        else:
            from paper_2203_05705_amd import workloads as WL
            wl = WL.conv_layer()
            A, Wt = (ard.to_device(wl.arrays[k]) for k in ("A", "Wt"))
            N, C, H, W = A.shape
            ws = torch.empty(ard.conv_workspace_bytes(ard.BF16, N, C, H, W, 256, 3, 3, 1, 1), dtype=torch.uint8, device="cuda")
            sel = ard.conv_select(A, 0.5, ws=ws)
            nk = int(sel["count"].item())
            Y = ard.conv_fwd(A, Wt, sel["keep"], nk, ws=ws)
            fn = lambda: ard.conv_fwd(A, Wt, sel["keep"], nk, ws=ws, out=Y)
        # timed as in the full run (bursts of 20 launches); no spin-up burst in front: 0.3 s of dense products
        # right before these large kernels leaves the chip at a lower clock than the full run finds it at
        t = event_us(torch, fn)
        print(json.dumps({"call": name, "launches": 5 + 20 * REPEATS, "avg_us": t["median"]}))
        return
    _, cdf = ard.search_k(0.5, N_PATTERNS)
    n_plan = max(100, args.steps + args.warmup)
    pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(n_plan)]
    plans = [chain.plan(pp) for pp in pats]
    used = [plans[(args.warmup + it) % len(plans)] for it in range(args.steps)]
    tot, cnt, fl = per_call_times(torch, chain, used, only=name)
    print(json.dumps({"call": name, "launches": cnt[name] * 4, "avg_us": tot[name] / cnt[name] * 1e3,
                      "kept_tflops": fl[name] / (tot[name] / 1e3) / 1e12}))


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
    if args.only_call not in ("C3.fwd.dp2", "C5.fwd"):
        spin_up(torch)

    if args.only_call:
        only_call(args, ard, torch, chain)
        return

    steps = args.steps
    # dense chains: this library at dp=1, and the vendor GEMM, run the same way as the dropout chain
    dense_plan = [chain.plan(((1, 1), (1, 1)))]
    t_lib_dense = time_steps(torch, chain, dense_plan, steps, args.warmup, args.mode)
    t_vendor = {m: time_torch_dense(torch, chain, steps, args.warmup, m) for m in ("eager", "graph")}
    t_lib_dense_eager = time_steps(torch, chain, dense_plan, steps, args.warmup, "eager")
    t_vendor_dense = min(v["median"] for v in t_vendor.values())
    t_dense = min(t_lib_dense["median"], t_vendor_dense)

    rates, headline, roof = {}, None, None
    rooflines = []
    cdf05 = None
    for p in (0.3, 0.5, 0.7):
        _, cdf = ard.search_k(p, N_PATTERNS)
        if p == 0.5:
            cdf05 = cdf
        pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(n_plan)]
        plans = [chain.plan(pp) for pp in pats]
        t = time_steps(torch, chain, plans, steps, args.warmup, args.mode)
        dt = t["median"]
        used = [plans[(args.warmup + it) % len(plans)] for it in range(steps)]
        kept_f = sum(c[5] for plan in used for c in chain.calls(plan)) / steps
        rates[str(p)] = dict(ms_per_step=dt * 1e3, ms_per_step_min=t["min"] * 1e3, ms_per_step_max=t["max"] * 1e3,
                             effective_tflops=dense_f / dt / 1e12, kept_tflops=kept_f / dt / 1e12,
                             speedup_vs_lib_dense=t_lib_dense["median"] / dt, speedup_vs_vendor_dense=t_vendor_dense / dt,
                             speedup_vs_dense=t_dense / dt, ideal_speedup_kept_flops=dense_f / kept_f,
                             target_speedup=1.0 / (1.0 - p))
        if p == 0.5:
            headline = t
            for other in ("grouped", "eager", "graph", "graph1"):
                if other != args.mode:
                    rates[str(p)][f"{other}_ms_per_step"] = time_steps(torch, chain, plans, steps, args.warmup, other)["median"] * 1e3
            cplans = [chain.plan(pp, compact_dw=True) for pp in pats]
            rates[str(p)]["compact_dw_ms_per_step"] = time_steps(torch, chain, cplans, steps, args.warmup, args.mode)["median"] * 1e3
            # roofline of the call that takes the largest share of the iteration, over the timed plans
            tot, cnt, fl = per_call_times(torch, chain, used)
            name = max(tot, key=tot.get)
            launch_us = tot[name] / cnt[name] * 1e3
            algo = sum(chain.algorithmic_bytes(plan, name) for plan in used) / len(used)
            roof = roofline_record(name, f"gemm_direct_kernel ({name}; the call's finishing pass, where it has one, included)",
                                   fl[name] / cnt[name], algo, launch_us, cnt[name] * 3)
            roof["per_call_avg_us"] = {k: round(v / cnt[k] * 1e3, 2) for k, v in tot.items()}
            lv, lcnt = per_level_times(torch, chain, used)
            roof["per_level_grouped_avg_us"] = lv
            roof["per_level_plans"] = lcnt
    dt = headline["median"]
    result = {
        "metric": "effective TFLOP/s + speedup vs dense GEMM at dropout 0.3/0.5/0.7, 1 MI355X",
        "value": dense_f / dt / 1e12, "unit": "effective TFLOP/s (dense-equivalent FLOPs / time) at rate 0.5",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": dt * 1e3,
        "ms_per_step_min": headline["min"] * 1e3, "ms_per_step_max": headline["max"] * 1e3, "repeats": REPEATS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "MLP 784-2048-2048-10, batch 1024, bf16 in / fp32 accumulate, row-based dropout on both "
                               "hidden layers, pattern per iteration from the searched distribution (N=8); fwd + bwd",
                   "rate": 0.5, "seed": SEED, "timing": f"median of {REPEATS} blocks of `steps` iterations",
                   "execution": {"graph": "one HIP-graph replay per iteration, weight gradients on a second lane",
                                 "eager": "calls issued one by one on one stream",
                                 "graph1": "one single-lane HIP-graph replay of the grouped launches per iteration",
                                 "grouped": "one stream; the independent calls of each of the iteration's 5 dependency levels "
                                            "issued as one grouped launch"}[args.mode]},
        "dense_ms_per_step": {"libard_dp1": t_lib_dense["median"] * 1e3, "libard_dp1_min": t_lib_dense["min"] * 1e3,
                              "libard_dp1_calls_one_by_one": t_lib_dense_eager["median"] * 1e3,
                              "vendor_torch_matmul_eager": t_vendor["eager"]["median"] * 1e3,
                              "vendor_torch_matmul_graph": t_vendor["graph"]["median"] * 1e3},
        "rates": rates, "roofline": roof,
    }
    if not args.no_extra:
        extra = {"tile_gemm_4096_bf16_tile64": extra_tile_gemm(ard, torch, rooflines),
                 "conv_fmap_drop_128x256x28x28_bf16": extra_conv(ard, torch, rooflines),
                 "lstm_1024_1024_b128_t64_bf16": extra_lstm(ard, torch),
                 "small_and_hbm_bound": extra_small(ard, torch),
                 "table1_mlp_sweep_batch128_rate0.7": extra_table1(ard, torch),
                 "lstm_1500_t35_batch_scaling": extra_lstm_batch_scaling(ard, torch)}
        result["roofline_large_shapes"] = rooflines
        result["extra"] = extra
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, cdf05, budget_s=12.0)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
