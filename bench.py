#!/usr/bin/env python3
"""Benchmark of the Metis split-FP4 linear hot path on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic input already
resident in HBM: every operand of every linear of the workload is decomposed
(metis_decompose) and split-quantized (metis_split_quantize), then the FP4 GEMMs run.
Default workload "c5": one LLaMA-3-8B layer's seven linears at 16384 tokens, each an
independent (X, W, G) triple: 21 decompositions + splits (both block orientations) and
21 GEMMs (fprop, dgrad, wgrad), 21.44 TFLOP of useful GEMM work per step.  "c1".."c4" are
the smaller configurations (c4 = the FFN down projection alone, full W4A4G4 step).

Prints ONE JSON line: whole-step throughput (useful GEMM flops / step time), the roofline
of the dominant kernel (the FP4 GEMM, HIP events around each of its launches inside the
timed region), the steady-state step in which weights are stored as parts (no weight
decomposition), per-pass HBM rates warm and cold, end-to-end effective bandwidth of
decompose + split against the algorithmic minimum, measured copy / read / matrix-loop
ceilings of the box, and the fp64 oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0     # MI355X dense fp16/bf16 matrix peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
PEAK_FP4_TFLOPS = 10100.0     # MI355X dense fp4/fp6 matrix peak

WORKLOAD_TEXT = {
    "c1": "config 1: tiny planted W 256x512 (k=8, p=8, rho=0.25) x X 128x512, decompose+split_quantize(W), quantize(X), fwd",
    "c2": "config 2: LLaMA-3-8B attention projection W 4096x4096 (k=64, p=16) x X 8192x4096, "
          "decompose+split_quantize(W), quantize(X), fwd",
    "c3": "config 3: FFN up W 14336x4096, X 8192x4096, both decomposed and split, fwd",
    "c4": "config 4: FFN down W 4096x14336, X 8192x14336, G 8192x4096, all decomposed and split both ways, "
          "fwd + dgrad + wgrad",
    "c5": "config 5: one LLaMA-3-8B layer at 16384 tokens, seven linears (q, o 4096x4096; k, v 1024x4096; gate, up "
          "14336x4096; down 4096x14336), each an independent (X, W, G) triple: 21 decompose + split_quantize (both "
          "orientations), 21 GEMMs (fwd + dgrad + wgrad)",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed step and its roofline (keeps a profile to the step's own kernels)")
    ap.add_argument("--fused", action="store_true",
                    help="decompose + split through the fused metis_decompose_split_quantize path (A read once from HBM, "
                         "band by band) instead of two calls per operand; measured slower on this GPU, hence not the default")
    ap.add_argument("--prep-streams", type=int, default=3,
                    help="streams the operands' decompositions and splits are spread over (they are independent of one "
                         "another; the GEMMs always run on the main stream after a join)")
    ap.add_argument("--no-phased-gemms", action="store_true",
                    help="with several streams: keep each GEMM's pre-pass directly in front of its main kernel instead of "
                         "running all pre-passes side by side first")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference dispatch for HBM byte counters)")
    return ap.parse_args()


class Operand:
    """One matrix of a linear with everything its decomposition and split need, preallocated."""

    def __init__(self, metis, torch, A, k, p, rho, seed, want_t):
        self.A = A.cuda()
        self.M, self.N = A.shape
        self.k, self.p, self.rho, self.seed, self.want_t = k, p, rho, seed, want_t
        g_r = metis.tensor_scale(float(A.abs().max()))           # delayed scaling: amax known from setup
        dev = "cuda"
        if k:
            self.U = torch.empty((self.M, k), dtype=torch.float32, device=dev)
            self.S = torch.empty((k,), dtype=torch.float32, device=dev)
            self.V = torch.empty((self.N, k), dtype=torch.float32, device=dev)
            self.ws_dec = torch.empty((metis.decompose_split_workspace_bytes(self.M, self.N, k, p, rho),),
                                      dtype=torch.uint8, device=dev)
            self.ws_split = torch.empty((metis.split_workspace_bytes(self.M, self.N, k),), dtype=torch.uint8, device=dev)
        self.q = metis.SplitTensor(self.M, self.N, k, 2.0 ** -11, 2.0 ** -11, g_r, want_t)
        self.metis, self.torch = metis, torch
        self.parts = None

    def decompose(self, rho=None):
        self.metis.decompose(self.A, self.k, self.p, self.rho if rho is None else rho, self.seed,
                             workspace=self.ws_dec, out=(self.U, self.S, self.V))

    def split(self):
        self.metis.split_quantize(self.A, self.U, self.S, self.V, self.q, workspace=self.ws_split)

    def fused(self):
        self.metis.decompose_split_quantize(self.A, self.k, self.p, self.rho, self.seed, self.q, workspace=self.ws_dec,
                                            factors=(self.U, self.S, self.V))

    def prepare(self, two_call=True):
        if self.k and not two_call:
            self.fused()
        elif self.k:
            self.decompose()
            self.split()
        else:
            self.metis.quantize(self.A, self.q.R, self.q.Rt)

    def store_parts(self):
        """Residual of the current factors as a stored bf16 variable (Sec. 3.2: a weight's factors and residual
        are separate parameters); set-up only."""
        t = self.torch
        self.parts = (self.A.float() - (self.U * self.S) @ self.V.T).to(t.bfloat16)

    def prepare_from_parts(self):
        self.metis.split_from_parts(self.parts, self.U, self.S, self.V, self.q)

    def orientations(self):
        return 2 if self.want_t else 1

    def min_bytes(self):
        """Algorithmic minimum of decompose + split: A read once, codes and scales written once per orientation."""
        return (2.0 + 0.5625 * self.orientations()) * self.M * self.N


class Linear:
    def __init__(self, name, W, X, G, metis, torch):
        self.name, self.W, self.X, self.G = name, W, X, G
        self.L, self.K, self.N = X.M, X.N, W.M
        kmax = max(W.k, X.k, G.k if G else 0)
        nbytes = max(metis.linear_workspace_bytes(self.L, self.N, self.K, kmax), 256)
        # one workspace per product, so that the pre-passes of all products can run before the first main kernel
        self.wss = [torch.empty((nbytes,), dtype=torch.uint8, device="cuda") for _ in range(3 if G else 1)]
        self.ws = self.wss[0]
        self.Y = torch.empty((self.L, self.N), dtype=torch.bfloat16, device="cuda")
        self.dX = torch.empty((self.L, self.K), dtype=torch.bfloat16, device="cuda") if G else None
        self.dW = torch.empty((self.N, self.K), dtype=torch.bfloat16, device="cuda") if G else None
        self.metis = metis

    def ops(self):
        return [o for o in (self.W, self.X, self.G) if o is not None]

    def n_gemms(self):
        return 3 if self.G else 1

    def flops(self):
        return 2.0 * self.L * self.K * self.N * self.n_gemms()

    def calls(self):
        """(product, a, b, out, workspace) of this linear's GEMMs."""
        m = self.metis
        c = [(m.LINEAR_FWD, self.X.q, self.W.q, self.Y, self.wss[0])]
        if self.G:
            c.append((m.LINEAR_DGRAD, self.G.q, self.W.q, self.dX, self.wss[1]))
            c.append((m.LINEAR_WGRAD, self.G.q, self.X.q, self.dW, self.wss[2]))
        return c

    def gemms(self):
        m = self.metis
        m.fp4_linear_fwd(self.X.q, self.W.q, self.Y, self.ws)
        if self.G:
            m.fp4_linear_dgrad(self.G.q, self.W.q, self.dX, self.ws)
            m.fp4_linear_wgrad(self.G.q, self.X.q, self.dW, self.ws)


def build_workload(name, metis, torch, workloads):
    c = int(name[1])
    prm = workloads.PARAMS[c]
    k, p = prm["k"], prm["p"]
    if c <= 4:
        T = workloads.config(c)
        full = c == 4
        W = Operand(metis, torch, T["W"], k, p, prm["rho_w"], workloads.seed_for(c, 0) + 7, full)
        X = Operand(metis, torch, T["X"], k if c >= 3 else 0, p, prm["rho_x"], workloads.seed_for(c, 1) + 7, full)
        G = Operand(metis, torch, T["G"], k, p, prm["rho_x"], workloads.seed_for(c, 2) + 7, True) if full else None
        return [Linear({1: "tiny", 2: "attn", 3: "ffn_up", 4: "ffn_down"}[c], W, X, G, metis, torch)], {"c": T}
    lin, host = [], {}
    for nm, _, _ in workloads.LAYER_LINEARS:
        T = workloads.layer_linear(nm)
        W = Operand(metis, torch, T["W"], k, p, prm["rho_w"], workloads.layer_seed(nm, "W"), True)
        X = Operand(metis, torch, T["X"], k, p, prm["rho_x"], workloads.layer_seed(nm, "X"), True)
        G = Operand(metis, torch, T["G"], k, p, prm["rho_x"], workloads.layer_seed(nm, "G"), True)
        lin.append(Linear(nm, W, X, G, metis, torch))
        if nm == "k":
            host["k"] = T                                           # the CPU baseline's sample
    return lin, host


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2509_00404_amd import metis, workloads
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    metis.lib()

    t0 = time.time()
    linears, host = build_workload(args.workload, metis, torch, workloads)
    setup_s = time.time() - t0
    all_ops = [o for l in linears for o in l.ops()]
    n_gemm = sum(l.n_gemms() for l in linears)
    n_split = sum(1 for o in all_ops if o.k)
    useful_flops = sum(l.flops() for l in linears)

    # One step: every decomposition in batched calls (the single-workgroup factorizations of the operands then run
    # side by side), the splits, then the GEMMs.  The operands are independent of one another until the GEMMs, so
    # their preparation is dealt over --prep-streams streams that the main stream joins before the first GEMM.
    split_ops = [o for o in all_ops if o.k]
    multi = n_split >= 2

    fused = args.fused

    def batch_of(ops):
        return metis.DecomposeBatch([dict(A=o.A, k=o.k, p=o.p, rho=o.rho, seed=o.seed, U=o.U, S=o.S, V=o.V,
                                          workspace=o.ws_dec, split=o.q if fused else None) for o in ops]) if ops else None

    batch_all = batch_of(split_ops)
    xg_ops = [o for l in linears for o in (l.X, l.G) if o is not None and o.k]
    batch_xg = batch_of(xg_ops)

    # Optional: the operands' preparation spread over several streams (default priority), largest operands dealt
    # round-robin; each stream runs its own batched decomposition and its splits, the main stream waits for all.
    n_prep = max(1, min(args.prep_streams, len(split_ops))) if multi else 1
    side = [torch.cuda.Stream() for _ in range(n_prep)] if n_prep > 1 else []
    fork = torch.cuda.Event() if side else None
    joins = [torch.cuda.Event() for _ in side]

    def deal(ops):
        groups = [[] for _ in range(n_prep)]
        for i, o in enumerate(sorted(ops, key=lambda o: -o.M * o.N)):
            groups[i % n_prep].append(o)
        return groups

    groups_all = [(g, batch_of(g)) for g in deal(split_ops)] if side else []
    groups_xg = [(g, batch_of(g)) for g in deal(xg_ops)] if side else []

    def prepare_ops(ops, lin_w, weights_from_parts):
        for o in ops:
            if not o.k:
                o.prepare()
            elif weights_from_parts and o in lin_w:
                o.prepare_from_parts()
            elif not fused:
                o.split()

    def step(weights_from_parts=False, streams=True):
        lin_w = [l.W for l in linears]
        use_side = side if streams else []
        if use_side:
            main_stream = torch.cuda.current_stream()
            fork.record(main_stream)
            groups = groups_xg if weights_from_parts else groups_all
            for st, ev, (ops, b) in zip(side, joins, groups):
                st.wait_event(fork)
                with torch.cuda.stream(st):
                    if b is not None:
                        b.run()
                    prepare_ops(ops, lin_w, False)
                    ev.record(st)
            # what is not decomposed in this step (plain operands, weights taken from their stored parts)
            rest = [o for o in all_ops if not o.k or (weights_from_parts and o in lin_w)]
            prepare_ops(rest, lin_w, weights_from_parts)
            for ev in joins:
                main_stream.wait_event(ev)
        else:
            b = batch_xg if weights_from_parts else batch_all
            if b is not None:
                b.run()
            prepare_ops(all_ops, lin_w, weights_from_parts)
        if use_side and not args.no_phased_gemms:
            # the pre-passes of all products (small kernels) side by side on the streams, then the main kernels back
            # to back on the main stream
            main_stream = torch.cuda.current_stream()
            calls = [c for l in linears for c in l.calls()]
            fork.record(main_stream)
            for i, (st, ev) in enumerate(zip(side, joins)):
                st.wait_event(fork)
                with torch.cuda.stream(st):
                    for prod, a, b, out, ws in calls[i::n_prep]:
                        metis.fp4_linear_phase(prod, metis.LINEAR_PREPARE, a, b, None, ws)
                    ev.record(st)
            for ev in joins:
                main_stream.wait_event(ev)
            for prod, a, b, out, ws in calls:
                metis.fp4_linear_phase(prod, metis.LINEAR_APPLY, a, b, out, ws)
        else:
            for l in linears:
                l.gemms()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones((1 << 28,), dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    timers = {
        "gemm": metis.KernelTimer(metis.PROF_GEMM, args.steps * n_gemm),
        "broadcast": metis.KernelTimer(metis.PROF_BROADCAST, max(1, args.steps * n_split)),
        "residual_quant": metis.KernelTimer(metis.PROF_RESIDUAL_QUANT, max(1, args.steps * n_split)),
        "quantize": metis.KernelTimer(metis.PROF_QUANTIZE, max(1, args.steps * 4)),
    }
    for t in timers.values():
        t.__enter__()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    for t in timers.values():
        t.__exit__()
    ms_per_step = elapsed * 1e3 / args.steps
    value = useful_flops / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the FP4 GEMM.  achieved = algorithmic flops of the bracketed launches / their summed durations
    gd = timers["gemm"].durations_ms(args.steps * n_gemm)
    gemm_ms = sum(gd) / len(gd)
    gemm_tflops = useful_flops * args.steps / (sum(gd) * 1e-3) / 1e12
    roofline = {"kernel": "k_fp4_gemm_nt_pipe", "bound": "mfma", "achieved": round(gemm_tflops, 2),
                "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_MFMA_TFLOPS, 4),
                "traffic": traffic_from_profile(args.workload), "avg_launch_ms": round(gemm_ms, 4),
                "launches_per_step": n_gemm, "flop_per_launch": useful_flops / n_gemm,
                "frac_of_fp8_peak": round(gemm_tflops / 5000.0, 4), "frac_of_fp4_peak": round(gemm_tflops / PEAK_FP4_TFLOPS, 4),
                "timing": "HIP events on the launch stream around every launch of the timed steps"}

    pass_steps = args.steps
    if n_prep > 1 and n_split:
        # with several preparation streams a launch shares the chip with the kernels of other operands, so its elapsed
        # time is not a rate of the kernel alone: the passes are timed on the same step replayed on one stream
        for name in ("broadcast", "residual_quant", "quantize"):
            timers[name].close()
        pass_steps = 3
        timers["broadcast"] = metis.KernelTimer(metis.PROF_BROADCAST, pass_steps * n_split)
        timers["residual_quant"] = metis.KernelTimer(metis.PROF_RESIDUAL_QUANT, pass_steps * n_split)
        timers["quantize"] = metis.KernelTimer(metis.PROF_QUANTIZE, max(1, pass_steps * 4))
        step(streams=False)
        torch.cuda.synchronize()
        for name in ("broadcast", "residual_quant", "quantize"):
            timers[name].__enter__()
        for _ in range(pass_steps):
            step(streams=False)
        torch.cuda.synchronize()
        for name in ("broadcast", "residual_quant", "quantize"):
            timers[name].__exit__()
    passes = {"note": ("the step replayed on one stream after the timed region (in the timed step the operands are prepared "
                       "on %d streams at once and a launch shares the chip with kernels of other operands)" % n_prep
                       if n_prep > 1 else "inside the timed step")
                      + "; per-shape figures, warm and cold, under passes_standalone"}
    if n_split:
        bd = timers["broadcast"].durations_ms(pass_steps * n_split)
        rd = timers["residual_quant"].durations_ms(pass_steps * n_split)
        bc_bytes = sum(2.0 * o.M * o.N for o in all_ops if o.k) * pass_steps
        rq_bytes = sum(o.min_bytes() for o in all_ops if o.k) * pass_steps
        passes["broadcast"] = rate(bc_bytes, sum(bd))
        passes["residual_quant"] = rate(rq_bytes, sum(rd))
    plain = [o for o in all_ops if not o.k]
    if plain:
        qd = timers["quantize"].durations_ms(pass_steps * len(plain))
        passes["quantize"] = rate(sum(2.5625 * o.M * o.N for o in plain) * pass_steps, sum(qd))
    for t in timers.values():
        t.close()

    out = {
        "metric": "split-FP4 linear TFLOP/s + decompose/quantize GB/s (frac of roofline), 1 GPU",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4(e2m1)+e4m3 block scales, fp16 MFMA, fp32 accumulate", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload],
                   "linears": [{"name": l.name, "L": l.L, "K": l.K, "N": l.N} for l in linears],
                   "k": all_ops[0].k or linears[0].W.k, "p": linears[0].W.p, "gemms_per_step": n_gemm,
                   "decompositions_per_step": n_split, "useful_tflop_per_step": round(useful_flops / 1e12, 3),
                   "prep_streams": n_prep,
                   "split_path": "fused decompose + split (one HBM pass over each operand, metis_decompose_batch)" if fused
                                 else "two calls per operand (metis_decompose_batch, then metis_split_quantize)",
                   "setup_s": round(setup_s, 1)},
        "roofline": roofline,
        "passes": passes,
    }

    if not args.no_extras:
        extras(out, args, torch, metis, linears, all_ops, step, multi, useful_flops)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, torch, workloads, host, args.workload)
    print(json.dumps(out))


def rate(nbytes, ms):
    gbs = nbytes / ms / 1e6
    return {"total_ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}


def timed(torch, fn, reps=5, between=None):
    """Wall time per call on the current stream, HIP events; `between` runs untimed before every call."""
    fn()                                          # kernels that no step has launched yet load on first use
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        if between:
            between()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    return {"median_ms": round(statistics.median(ts), 4), "min_ms": round(min(ts), 4)}


def extras(out, args, torch, metis, linears, all_ops, step, multi, useful_flops):
    """Figures beside the timed step; none of them enters `value`."""
    # steady state (Sec. 3.2): the weights' factors and residuals are stored variables, so a training step
    # quantizes them as they are (metis_split_from_parts); activations and gradients are decomposed every step
    if multi:
        for l in linears:
            l.W.store_parts()
        for _ in range(2):
            step(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(True)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["steady_state"] = {"what": "weights quantized from stored parts (no weight decomposition); X and G decomposed",
                               "ms_per_step": round(ms, 4), "value": round(useful_flops / (ms * 1e-3) / 1e12, 3),
                               "unit": "TFLOP/s"}
        for l in linears:
            l.W.parts = None
        step()                                     # back to the decomposed weights' codes
        torch.cuda.synchronize()

    # measured ceilings of this machine (library kernels metis_ceiling_*)
    buf_a = torch.empty((1 << 29,), dtype=torch.uint8, device="cuda")
    buf_b = torch.empty((1 << 29,), dtype=torch.uint8, device="cuda")
    buf_a.fill_(1)
    sink = torch.zeros((512 * 256,), dtype=torch.float32, device="cuda")
    tc = timed(torch, lambda: metis.ceiling_copy(buf_a, buf_b))
    tr = timed(torch, lambda: metis.ceiling_read(buf_a, sink.view(torch.int32)))
    # (launches of several milliseconds: a sub-millisecond launch after an idle gap runs at a lower clock)
    fl = metis.ceiling_mfma(20000, sink)
    tm = timed(torch, lambda: metis.ceiling_mfma(20000, sink))
    out["ceilings"] = {
        "copy_GB/s": round(2 * buf_a.numel() / tc["median_ms"] / 1e6, 1),
        "read_GB/s": round(buf_a.numel() / tr["median_ms"] / 1e6, 1),
        "mfma_fp16_loop_TFLOP/s": round(fl / (tm["median_ms"] * 1e-3) / 1e12, 1),
        "what": "512 MiB streaming copy and read (beyond the 256 MB last-level cache), register-resident 32x32x16 fp16 "
                "matrix-instruction loop on all CUs (2 waves per SIMD, ~%.0f ms)" % tm["median_ms"]}

    # the GEMM's instruction mix without its memory system: matrix instructions with N packed multiplies each
    mix = {}
    for wps in (1, 2):
        for nv in (0, 4, 5, 6, 8):
            flm = metis.ceiling_mfma_mix(50000, nv, wps, sink)
            tmix = timed(torch, lambda: metis.ceiling_mfma_mix(50000, nv, wps, sink))
            mix["%d wave%s per SIMD, %d multiplies per matrix instruction" % (wps, "s" if wps > 1 else "", nv)] = round(
                flm / (tmix["median_ms"] * 1e-3) / 1e12, 1)
    out["ceilings"]["mfma_fp16_with_vector_work_TFLOP/s"] = mix
    # the GEMM's own expansion and matrix instructions on registers: the stage loop without LDS, loads, waits, barrier
    fle = metis.ceiling_mfma_mix(20000, metis.MIX_GEMM_EXPANSION, 1, sink)
    te = timed(torch, lambda: metis.ceiling_mfma_mix(20000, metis.MIX_GEMM_EXPANSION, 1, sink))
    out["ceilings"]["gemm_stage_loop_on_registers_TFLOP/s"] = round(fle / (te["median_ms"] * 1e-3) / 1e12, 1)
    fl6 = metis.ceiling_mfma_mix(20000, metis.MIX_GEMM_EXPANSION_FP6, 1, sink)
    t6 = timed(torch, lambda: metis.ceiling_mfma_mix(20000, metis.MIX_GEMM_EXPANSION_FP6, 1, sink))
    out["ceilings"]["gemm_stage_loop_on_registers_fp6_containers_TFLOP/s"] = round(fl6 / (t6["median_ms"] * 1e-3) / 1e12, 1)

    def sweep():                                   # evicts the last-level cache: 1 GiB of other traffic
        metis.ceiling_copy(buf_a, buf_b)

    # stand-alone passes, one operand at a time, per distinct operand shape: warm (back to back) and cold (cache swept)
    seen, alone = set(), []
    for o in sorted((o for o in all_ops if o.k), key=lambda o: -o.M * o.N):
        key = (o.M, o.N, o.orientations(), o.rho)
        if key in seen or len(alone) >= 6:
            continue
        seen.add(key)
        row = {"shape": [o.M, o.N], "orientations": o.orientations(), "sample_rate": round(o.rho, 4)}
        mn = o.M * o.N
        for mode, two_call in (("two_call", True), ("fused", False)):
            row[mode] = {}
            for label, between in (("warm", None), ("cold", sweep)):
                nb = 7 * 16                                        # the fused path launches one pair of kernels per band
                tb = metis.KernelTimer(metis.PROF_BROADCAST, nb)
                tq = metis.KernelTimer(metis.PROF_RESIDUAL_QUANT, nb)
                tot = []
                o.prepare(two_call)
                torch.cuda.synchronize()
                with tb, tq:
                    for _ in range(7):
                        if between:
                            between()
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        o.prepare(two_call)
                        e1.record()
                        torch.cuda.synchronize()
                        tot.append(e0.elapsed_time(e1))
                bd, rd = tb.durations_ms(nb), tq.durations_ms(nb)
                tb.close()
                tq.close()
                bands = max(1, len(bd) // 7) if not two_call else 1
                bd = [sum(bd[i * bands:(i + 1) * bands]) for i in range(min(7, len(bd) // bands))]
                rd = [sum(rd[i * bands:(i + 1) * bands]) for i in range(min(7, len(rd) // bands))]
                row[mode][label] = {
                    "broadcast": dict(median_us=round(statistics.median(bd) * 1e3, 1), min_us=round(min(bd) * 1e3, 1),
                                      frac_hbm=round(2.0 * mn / statistics.median(bd) / 1e6 / PEAK_HBM_GBS, 4)),
                    "residual_quant": dict(median_us=round(statistics.median(rd) * 1e3, 1), min_us=round(min(rd) * 1e3, 1),
                                           frac_hbm=round(o.min_bytes() / statistics.median(rd) / 1e6 / PEAK_HBM_GBS, 4)),
                    "decompose_plus_split": dict(median_ms=round(statistics.median(tot), 4), min_ms=round(min(tot), 4),
                                                 effective_GBps_vs_minimum=round(o.min_bytes() / statistics.median(tot) / 1e6, 1))}
                if not two_call:
                    row[mode][label]["bands"] = bands
        alone.append(row)
    out["passes_standalone"] = {
        "rows": alone,
        "bytes": "broadcast 2 M N; residual_quant (2 + 0.5625 orientations) M N (in the fused path the band's second "
                 "read comes from the last-level cache; the fraction is still bytes moved / time); decompose_plus_split is "
                 "the whole chain against the algorithmic minimum 2 M N + 0.5625 M N orientations",
        "timing": "HIP event pairs (about 3 us of bracket overhead per kernel); cold = a 1 GiB copy between repetitions"}

    # per-call wall time of each entry point on the first linear (and the last, if different)
    phases = {}
    for l in ([linears[0]] if len(linears) == 1 else [linears[0], linears[-1]]):
        for nm, o in (("W", l.W), ("X", l.X), ("G", l.G)):
            if o is None:
                continue
            tag = f"{l.name}.{nm}[{o.M}x{o.N}]"
            if o.k:
                phases[f"decompose {tag}"] = timed(torch, o.decompose)
                phases[f"split_quantize {tag}"] = timed(torch, o.split)
            else:
                phases[f"quantize {tag}"] = timed(torch, o.prepare)
        phases[f"linear_fwd {l.name}"] = timed(torch, lambda: metis.fp4_linear_fwd(l.X.q, l.W.q, l.Y, l.ws))
        if l.G:
            phases[f"linear_dgrad {l.name}"] = timed(torch, lambda: metis.fp4_linear_dgrad(l.G.q, l.W.q, l.dX, l.ws))
            phases[f"linear_wgrad {l.name}"] = timed(torch, lambda: metis.fp4_linear_wgrad(l.G.q, l.X.q, l.dW, l.ws))
    # the paper's sampling rate ("less than 1 % of the rows"): one data point
    big = max((o for o in all_ops if o.k and o.rho < 1.0), key=lambda o: o.M * o.N, default=None)
    if big is not None:
        try:
            phases[f"decompose [{big.M}x{big.N}] at sample_rate 0.01"] = timed(torch, lambda: big.decompose(0.01))
            big.decompose()
        except metis.MetisError as e:
            phases["decompose at sample_rate 0.01"] = {"error": str(e)[:120]}
    l0 = linears[0]
    if l0.W.k and l0.G:
        gU = torch.empty((l0.N, l0.W.k), dtype=torch.float32, device="cuda")
        gS = torch.empty((l0.W.k, l0.W.k), dtype=torch.float32, device="cuda")
        gV = torch.empty((l0.K, l0.W.k), dtype=torch.float32, device="cuda")
        ws_fg = torch.empty((metis.factor_grads_workspace_bytes(l0.N, l0.K, l0.W.k),), dtype=torch.uint8, device="cuda")
        phases[f"factor_grads {l0.name}.W"] = timed(torch, lambda: metis.fp4_factor_grads(l0.dW, l0.W.q, gU, gS, gV, ws_fg))
    out["phases"] = phases

    # the same product in the MXFP4 variant (block 32, power-of-two scales that the matrix instruction applies itself)
    l = linears[-1]
    if l.K % 32 == 0:
        try:
            qx, qw = metis.MxTensor(l.L, l.K), metis.MxTensor(l.N, l.K)
            Ymx = torch.empty((l.L, l.N), dtype=torch.bfloat16, device="cuda")
            mx_q = timed(torch, lambda: (metis.quantize_mx(l.X.A, qx), metis.quantize_mx(l.W.A, qw)))
            mx_g = timed(torch, lambda: metis.mxfp4_gemm_nt(qx, qw, Ymx))
            tf = 2.0 * l.L * l.K * l.N / (mx_g["median_ms"] * 1e-3) / 1e12
            out["mxfp4_variant"] = {"kernel": "k_mxfp4_gemm_nt", "linear": l.name, "quantize_both_ms": mx_q["median_ms"],
                                    "gemm_ms": mx_g["median_ms"], "achieved": round(tf, 1), "peak": PEAK_FP4_TFLOPS,
                                    "unit": "TFLOP/s", "frac": round(tf / PEAK_FP4_TFLOPS, 4)}
        except Exception as e:                                     # an extra figure must never cost the main line
            out["mxfp4_variant"] = {"error": repr(e)[:200]}
    # stochastic rounding of the largest activation (the paper's training default; the timed step rounds to nearest)
    try:
        x = max((o for o in all_ops), key=lambda o: o.M * o.N)
        sr = timed(torch, lambda: metis.quantize_sr(x.A, 1, x.q.R, None))
        rn = timed(torch, lambda: metis.quantize(x.A, x.q.R, None))
        rh = timed(torch, lambda: metis.quantize_rht_sr(x.A, 1, x.q.R))
        qb = 2.5625 * x.M * x.N
        out["quantize_plain"] = {"shape": [x.M, x.N],
                                 "what": "plain quantizer of the largest operand, one orientation: nearest rounding, stochastic "
                                         "rounding, and the comparison recipe (random 16-point Hadamard rotation + stochastic rounding)",
                                 "nearest": dict(rn, frac_hbm=round(qb / rn["median_ms"] / 1e6 / PEAK_HBM_GBS, 4)),
                                 "stochastic": dict(sr, frac_hbm=round(qb / sr["median_ms"] / 1e6 / PEAK_HBM_GBS, 4)),
                                 "hadamard_stochastic": dict(rh, frac_hbm=round(qb / rh["median_ms"] / 1e6 / PEAK_HBM_GBS, 4))}
        x.prepare()
    except Exception as e:
        out["quantize_plain"] = {"error": repr(e)[:200]}


def traffic_from_profile(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel calibration); None if there is none."""
    path = os.path.join(ROOT, "profiles", f"bench_config{workload[1]}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("k_fp4_gemm_nt_pipe<unsigned short>"):
                tail = line[52:].split()
                return round((float(tail[0]) + float(tail[1])) * 2 ** 20)
    except OSError:
        pass
    return None


def cpu_baseline(np, torch, workloads, host, workload):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload (test infrastructure, timed only)."""
    from oracle import decompose as odec
    from oracle import linear as olin
    from oracle import quant as oq
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    c = int(workload[1])
    prm = workloads.PARAMS[c]
    k, p = prm["k"], prm["p"]
    T = host["k"] if c == 5 else host["c"]
    cap = 2048                                                     # tokens of the sample
    Wn = T["W"].double().numpy()
    Xn = T["X"][:cap].double().numpy()
    Gn = T["G"][:cap].double().numpy() if "G" in T else None
    split_x = c >= 3
    both = Gn is not None

    def sq(A, kk, rho, seed):
        g = oq.tensor_scale_for(np.abs(A).max())
        if kk:
            U, S, V = odec.decompose(A, kk, p, rho, seed)
            return olin.split_quantize(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, want_t=both)
        return olin.split_quantize(A, None, None, None, 1.0, 1.0, g, want_t=both)

    passes, t0, dt = 0, time.perf_counter(), 0.0
    while dt < 10.0 and passes < 64:
        wq = sq(Wn, k, prm["rho_w"], 1)
        xq = sq(Xn, k if split_x else 0, max(prm["rho_x"], (k + p) / Xn.shape[0]), 2)
        olin.linear_fwd(xq, wq)
        if both:
            gq = sq(Gn, k, max(prm["rho_x"], (k + p) / Gn.shape[0]), 3)
            olin.linear_dgrad(gq, wq)
            olin.linear_wgrad(gq, xq)
        passes += 1
        dt = time.perf_counter() - t0
    flops = 2.0 * Xn.shape[0] * Wn.shape[0] * Wn.shape[1] * (3 if both else 1) * passes
    what = "the k projection of the layer (W 1024x4096)" if c == 5 else f"the workload's linear (W {Wn.shape[0]}x{Wn.shape[1]})"
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": f"{passes} whole steps of {what} on the first {Xn.shape[0]} tokens: decompose + split_quantize of every "
                      f"split operand, {'fwd + dgrad + wgrad' if both else 'fwd'}; useful GEMM flops / oracle seconds"}


if __name__ == "__main__":
    main()
