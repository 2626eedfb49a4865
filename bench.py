#!/usr/bin/env python3
"""Benchmark of the Approximate Random Dropout hot path on one MI355X.

Headline workload (BASELINE config 2): MLP 784-2048-2048-10, batch 1024, bf16
inputs with fp32 accumulation, row-based dropout on both hidden layers, a new
pattern (dp, b) sampled per iteration and layer from the searched distribution.
One step = one training iteration: 3 forward GEMMs (ReLU fused), 3 weight-gradient
GEMMs and 2 data-gradient GEMMs (ReLU backward fused), all through libard's C ABI.

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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (cpu_baseline) leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    return ap.parse_args()


class MlpChain:
    """Device buffers and prebuilt C-ABI argument lists for the config-2 iteration."""

    def __init__(self, ard, torch, wl):
        to_dev = lambda a, _dt: ard.to_device(a)
        self.ard, self.torch = ard, torch
        self.lib = ard.lib()
        dt = torch.bfloat16
        self.X0 = to_dev(wl.arrays["X0"], "bf16")
        self.W = [to_dev(wl.arrays[f"W{l}"], "bf16") for l in (1, 2, 3)]
        self.dYL = to_dev(wl.arrays["dY"], "bf16")
        B = BATCH
        self.Y = [torch.empty((B, SIZES[l]), dtype=dt, device="cuda") for l in (1, 2, 3)]
        self.dYh = [torch.empty((B, SIZES[l]), dtype=dt, device="cuda") for l in (1, 2)]   # gradient at hidden outputs
        self.dW = [torch.empty_like(w) for w in self.W]
        self.Wc = [torch.empty(((w.shape[0] + 7) & ~7, (w.shape[1] + 7) & ~7), dtype=dt, device="cuda")
                   for w in self.W[1:]]   # kept blocks of W2, W3 (axes padded to multiples of 8)
        self.ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
        self.stream = torch.cuda.current_stream().cuda_stream
        self._keep = []

    def _pat(self, dp, b):
        p = self.ard.CPattern(self.ard.PAT_ROW, dp, b, 0, 0, 0, None, None, None, None, None)
        self._keep.append(p)
        return C.byref(p)

    def plan(self, pats):
        """pats = ((dp1,b1),(dp2,b2)) -> list of (fn, args, name, kept_flops).

        Hidden activations and their gradients stay compact between the calls (only kept
        neurons are stored); W2's kept block is gathered once per iteration and shared by the
        forward and the data-gradient product; weight gradients are written in full."""
        lib, B, s, ws = self.lib, BATCH, self.stream, self.ws
        p1, p2 = self._pat(*pats[0]), self._pat(*pats[1])
        k1 = -(-(SIZES[1] - (pats[0][1] - 1)) // pats[0][0])
        k2 = -(-(SIZES[2] - (pats[1][1] - 1)) // pats[1][0])
        X0, (W1, W2, W3), (Y1, Y2, Y3), (dY1, dY2), (dW1, dW2, dW3) = self.X0, self.W, self.Y, self.dYh, self.dW
        W2c, W3c = self.Wc
        bf = self.ard.BF16
        IN, OUT, WC = self.ard.IN_COMPACT, self.ard.OUT_COMPACT, self.ard.W_COMPACT
        P = lambda t: t.data_ptr()
        f = 2.0 * B
        n = ws.numel()
        calls = [
            (lib.ard_drop_gemm_fwd, (bf, B, SIZES[0], SIZES[1], P(X0), P(W1), P(Y1), p1, None, 1.0, 1, OUT, P(ws), n, s), "L1.fwd", f * SIZES[0] * k1),
            (lib.ard_compact_weight, (bf, SIZES[1], SIZES[2], P(W2), P(W2c), p2, p1, s), "L2.compact_w", 0.0),
            (lib.ard_drop_gemm_fwd, (bf, B, SIZES[1], SIZES[2], P(Y1), P(W2c), P(Y2), p2, p1, 1.0, 1, IN | OUT | WC, P(ws), n, s), "L2.fwd", f * k1 * k2),
            (lib.ard_compact_weight, (bf, SIZES[2], SIZES[3], P(W3), P(W3c), None, p2, s), "L3.compact_w", 0.0),
            (lib.ard_drop_gemm_fwd, (bf, B, SIZES[2], SIZES[3], P(Y2), P(W3c), P(Y3), None, p2, 1.0, 0, IN | WC, P(ws), n, s), "L3.fwd", f * k2 * SIZES[3]),
            (lib.ard_drop_gemm_bwd_weight, (bf, B, SIZES[2], SIZES[3], P(self.dYL), P(Y2), P(dW3), None, p2, 1.0, 0.0, IN, P(ws), n, s), "L3.bwd_weight", f * k2 * SIZES[3]),
            (lib.ard_drop_gemm_bwd_data, (bf, B, SIZES[2], SIZES[3], P(self.dYL), P(W3c), P(dY2), None, p2, 1.0, P(Y2), IN | WC, P(ws), n, s), "L3.bwd_data", f * k2 * SIZES[3]),
            (lib.ard_drop_gemm_bwd_weight, (bf, B, SIZES[1], SIZES[2], P(dY2), P(Y1), P(dW2), p2, p1, 1.0, 0.0, IN | OUT, P(ws), n, s), "L2.bwd_weight", f * k1 * k2),
            (lib.ard_drop_gemm_bwd_data, (bf, B, SIZES[1], SIZES[2], P(dY2), P(W2c), P(dY1), p2, p1, 1.0, P(Y1), IN | OUT | WC, P(ws), n, s), "L2.bwd_data", f * k1 * k2),
            (lib.ard_drop_gemm_bwd_weight, (bf, B, SIZES[0], SIZES[1], P(dY1), P(X0), P(dW1), p1, None, 1.0, 0.0, OUT, P(ws), n, s), "L1.bwd_weight", f * SIZES[0] * k1),
        ]
        return calls

    def torch_dense_step(self):
        t = self.torch
        X0, (W1, W2, W3) = self.X0, self.W
        Y1 = t.relu(X0 @ W1.t())
        Y2 = t.relu(Y1 @ W2.t())
        Y3 = Y2 @ W3.t()  # noqa: F841
        dW3 = self.dYL.t() @ Y2  # noqa: F841
        dY2 = (self.dYL @ W3) * (Y2 > 0)
        dW2 = dY2.t() @ Y1  # noqa: F841
        dY1 = (dY2 @ W2) * (Y1 > 0)
        dW1 = dY1.t() @ X0  # noqa: F841


def dense_flops_per_iter():
    f = 2.0 * BATCH
    l1, l2, l3 = SIZES[0] * SIZES[1], SIZES[1] * SIZES[2], SIZES[2] * SIZES[3]
    return f * (2 * l1 + 3 * l2 + 3 * l3)      # fwd x3, dW x3, dX for L2 and L3


def run_calls(calls):
    for fn, args, _, _ in calls:
        rc = fn(*args)
        if rc != 0:
            raise RuntimeError(f"libard call failed with {rc}")


def time_steps(torch, plans, steps, warmup, bracket=None):
    """Run warmup + exactly `steps` iterations; returns (seconds, bracketed kernel ms list)."""
    n = len(plans)
    for it in range(warmup):
        run_calls(plans[it % n])
    torch.cuda.synchronize()
    evs = []
    t0 = time.perf_counter()
    for it in range(steps):
        calls = plans[(warmup + it) % n]
        if bracket is None:
            run_calls(calls)
        else:
            for fn, args, name, _ in calls:
                if name == bracket:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    fn(*args)
                    e1.record()
                    evs.append((e0, e1))
                else:
                    fn(*args)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, [a.elapsed_time(b) for a, b in evs]


def pick_dominant(torch, plans):
    """Untimed pre-pass: per-call HIP-event durations, summed per call name."""
    tot = {}
    for calls in plans[:min(20, len(plans))]:
        for fn, args, name, _ in calls:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(*args)
            e1.record()
            torch.cuda.synchronize()
            tot[name] = tot.get(name, 0.0) + e0.elapsed_time(e1)
    return max(tot, key=tot.get), tot


def cpu_baseline(wl, cdf, n_iter):
    """The oracle as it stands, timed on the host cores over a few iterations of the same workload."""
    import numpy as np
    from oracle import gemm as G
    from oracle import patterns as P
    from oracle import rounding as R
    from oracle import sampler as S
    X0 = wl.values("X0")
    Ws = [wl.values(f"W{l}") for l in (1, 2, 3)]
    dYL = wl.values("dY")
    t0 = time.perf_counter()
    for it in range(n_iter):
        pats = [S.sample_pattern(cdf, SEED, it, layer) for layer in (1, 2)]
        masks = [P.row_mask(SIZES[l + 1], *pats[l]) for l in range(2)]
        G.mlp_iteration(X0, Ws, dYL, masks, R.to_bf16_values)
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return dict(value=dense_flops_per_iter() * n_iter / dt / 1e12, unit="effective TFLOP/s", cores=threads,
                kind="oracle", sample=f"{n_iter} iterations of the config-2 MLP at target rate 0.5 (fp64 NumPy, masks materialised)",
                seconds=dt)


def extra_workloads(ard, torch):
    """Config 3 (tile pattern, 4096^3 bf16): per-GEMM times and speedups. Short by design."""
    out = {}
    n = 4096
    g = torch.Generator(device="cuda").manual_seed(3)
    X = torch.randn((n, n), generator=g, device="cuda").to(torch.bfloat16)
    W = (0.02 * torch.randn((n, n), generator=g, device="cuda")).to(torch.bfloat16)
    dY = torch.randn((n, n), generator=g, device="cuda").to(torch.bfloat16)
    outb = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")

    def t_us(fn, reps=10, warm=2):
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
    for dp in (1, 2, 3, 4):
        pat = ard.Pattern.tile(dp, 1, 64, 64)
        pat = ard.Pattern.tile(dp, 1, 64, 64, lists=ard.pattern_gen(pat, n, n))
        kept = int(pat.lists["count"].item())
        flops = 2.0 * n * 64 * 64 * kept
        row = {}
        for name, fn in (("fwd", lambda: ard.drop_gemm_fwd(X, W, pat, out=outb, ws=ws)),
                         ("bwd_data", lambda: ard.drop_gemm_bwd_data(dY, W, pat, out=outb, ws=ws)),
                         ("bwd_weight", lambda: ard.drop_gemm_bwd_weight(dY, X, pat, out=outb, ws=ws))):
            us = t_us(fn, reps=5, warm=1)
            row[name] = dict(us=round(us, 1), kept_tflops=round(flops / us / 1e6, 1),
                             frac_mfma_peak=round(flops / us / 1e6 / MFMA_PEAK_BF16, 4))
        res[f"dp{dp}"] = row
    for name in ("fwd", "bwd_data", "bwd_weight"):
        dense = min(vendor[name], res["dp1"][name]["us"])
        res["dp2"][name]["speedup_vs_dense"] = round(dense / res["dp2"][name]["us"], 3)
    out["tile_gemm_4096_bf16_tile64"] = res
    return out


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
    wl = WL.mlp_chain(seed=SEED, B=BATCH, sizes=SIZES)
    chain = MlpChain(ard, torch, wl)
    dense_f = dense_flops_per_iter()
    n_plan = max(100, args.steps + args.warmup)

    # dense chains: this library at dp=1, and the vendor GEMM
    dense_plan = [chain.plan(((1, 1), (1, 1)))]
    t_lib_dense, _ = time_steps(torch, dense_plan, args.steps, args.warmup)
    for _ in range(args.warmup):
        chain.torch_dense_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        chain.torch_dense_step()
    torch.cuda.synchronize()
    t_vendor_dense = time.perf_counter() - t0
    t_dense = min(t_lib_dense, t_vendor_dense)

    rates, headline, roof = {}, None, None
    cdf05 = None
    for p in (0.3, 0.5, 0.7):
        _, cdf = ard.search_k(p, N_PATTERNS)
        if p == 0.5:
            cdf05 = cdf
        pats = [tuple(ard.pattern_sample(cdf, SEED, it, layer) for layer in (1, 2)) for it in range(n_plan)]
        plans = [chain.plan(pp) for pp in pats]
        bracket = None
        if p == 0.5:
            bracket, per_call = pick_dominant(torch, plans)
        dt, kms = time_steps(torch, plans, args.steps, args.warmup, bracket)
        used = [plans[(args.warmup + it) % len(plans)] for it in range(args.steps)]
        kept_f = sum(c[3] for calls in used for c in calls)
        rates[str(p)] = dict(ms_per_step=dt / args.steps * 1e3, effective_tflops=dense_f * args.steps / dt / 1e12,
                             kept_tflops=kept_f / dt / 1e12, speedup_vs_lib_dense=t_lib_dense / dt,
                             speedup_vs_vendor_dense=t_vendor_dense / dt, speedup_vs_dense=t_dense / dt,
                             ideal_speedup=dense_f * args.steps / kept_f)
        if p == 0.5:
            headline = (dt, kept_f)
            kflops = sum(c[3] for calls in used for c in calls if c[2] == bracket)
            ksec = sum(kms) / 1e3
            roof = dict(bound="mfma", kernel=f"gemm_kernel ({bracket})", achieved=kflops / ksec / 1e12,
                        peak=MFMA_PEAK_BF16, unit="TFLOP/s", frac=kflops / ksec / 1e12 / MFMA_PEAK_BF16,
                        avg_launch_us=ksec / len(kms) * 1e6, traffic=None,
                        per_call_ms_prepass={k: round(v, 4) for k, v in per_call.items()})
    dt, _ = headline
    result = {
        "metric": "effective TFLOP/s + speedup vs dense GEMM at dropout 0.3/0.5/0.7, 1 MI355X",
        "value": dense_f * args.steps / dt / 1e12, "unit": "effective TFLOP/s (dense-equivalent FLOPs / time) at rate 0.5",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "MLP 784-2048-2048-10, batch 1024, bf16 in / fp32 accumulate, row-based dropout on both "
                               "hidden layers, pattern per iteration from the searched distribution (N=8); fwd + bwd",
                   "rate": 0.5, "seed": SEED},
        "dense_ms_per_step": {"libard_dp1": t_lib_dense / args.steps * 1e3, "vendor_torch_matmul": t_vendor_dense / args.steps * 1e3},
        "rates": rates, "roofline": roof,
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, cdf05, n_iter=6)
    if not args.no_extra:
        result["extra"] = extra_workloads(ard, torch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
