#!/usr/bin/env python3
"""Benchmark of the Metis split-FP4 linear hot path on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic input
already resident in HBM.  Default workload "c2": the LLaMA-3-8B attention projection
(W 4096x4096 decomposed with k=64, p=16 and split-quantized; X 8192x4096 quantized;
forward X W^T on the FP4 operands).  "c4" is the full W4A4G4 step of the FFN down
projection (three decompositions, three split-quantizations with both block
orientations, fprop + dgrad + wgrad).

Prints ONE JSON line: whole-step throughput (useful GEMM flops / step time), the
roofline of the dominant kernel (the FP4 GEMM, measured with HIP events around each of
its launches inside the timed region), per-pass HBM rates, and the fp64 oracle timed on
the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0     # MI355X dense fp16/bf16 matrix peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
PEAK_FP4_TFLOPS = 10100.0     # MI355X dense fp4/fp6 matrix peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ffn-passes", action="store_true",
                    help="skip the extra figure on an 8192 x 14336 operand (keeps a profile to the workload's own shapes)")
    ap.add_argument("--pipeline-depth", type=int, default=3,
                    help="extra measurement: independent steps in flight at once, one stream and one set of "
                         "buffers each (0 or 1 = skip); never enters `value`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference dispatch for HBM byte counters)")
    return ap.parse_args()


class Operand:
    """One matrix of the layer with everything its decomposition and split need, preallocated."""

    def __init__(self, metis, torch, A, k, p, rho, seed, want_t, oq, share=None):
        self.A = share.A if share is not None else A.cuda()       # a pipeline slot reads the same input
        self.M, self.N = A.shape
        self.k, self.p, self.rho, self.seed = k, p, rho, seed
        g_r = oq.tensor_scale_for(float(A.abs().max()))         # delayed scaling: amax known from setup
        dev = "cuda"
        if k:
            self.U = torch.empty((self.M, k), dtype=torch.float32, device=dev)
            self.S = torch.empty((k,), dtype=torch.float32, device=dev)
            self.V = torch.empty((self.N, k), dtype=torch.float32, device=dev)
            self.ws_dec = torch.empty((metis.decompose_workspace_bytes(self.M, self.N, k, p, rho),),
                                      dtype=torch.uint8, device=dev)
            self.ws_split = torch.empty((metis.split_workspace_bytes(self.M, self.N, k),), dtype=torch.uint8, device=dev)
        self.q = metis.SplitTensor(self.M, self.N, k, 2.0 ** -11, 2.0 ** -11, g_r, want_t)
        self.metis = metis

    def prepare(self):
        m = self.metis
        if self.k:
            m.decompose(self.A, self.k, self.p, self.rho, self.seed, workspace=self.ws_dec, out=(self.U, self.S, self.V))
            m.split_quantize(self.A, self.U, self.S, self.V, self.q, workspace=self.ws_split)
        else:
            m.quantize(self.A, self.q.R, self.q.Rt)

    def bytes_read_once(self):
        return 2 * self.M * self.N


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2509_00404_amd import metis, workloads
    from oracle import quant as oq                    # only tensor_scale_for (setup) and the cpu_baseline leg
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    metis.lib()

    c = int(args.workload[1])
    prm = workloads.PARAMS[c]
    t0 = time.time()
    T = workloads.config(c)
    k, p = prm["k"], prm["p"]
    split_x = c >= 3
    full = c == 4
    W = Operand(metis, torch, T["W"], k, p, prm["rho_w"], workloads.seed_for(c, 0) + 7, full, oq)
    X = Operand(metis, torch, T["X"], k if split_x else 0, p, prm["rho_x"], workloads.seed_for(c, 1) + 7, full, oq)
    G = Operand(metis, torch, T["G"], k, p, prm["rho_x"], workloads.seed_for(c, 2) + 7, True, oq) if full else None
    L, K = X.M, X.N
    N = W.M
    ws_lin = torch.empty((max(metis.linear_workspace_bytes(L, N, K, k), 256),), dtype=torch.uint8, device="cuda")
    Y = torch.empty((L, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((L, K), dtype=torch.bfloat16, device="cuda") if full else None
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda") if full else None
    setup_s = time.time() - t0
    ops = [W, X] + ([G] if full else [])
    n_gemm = 3 if full else 1

    # The operands' preparations (decompose + split_quantize, or quantize) are independent of each other, and
    # the decomposition's small-matrix kernels occupy one CU each: one stream per operand lets them overlap.
    # Every entry point only enqueues on the caller's current stream, so this is plain caller-side concurrency.
    main_stream = torch.cuda.current_stream()
    side = [torch.cuda.Stream() for _ in ops]                 # default priority
    ev_fork = torch.cuda.Event()
    ev_join = [torch.cuda.Event() for _ in ops]

    multi = sum(1 for o in ops if o.k) >= 2                   # worth a fork/join only with two or more decompositions

    def step():
        if not multi:
            for o in ops:
                o.prepare()
            metis.fp4_linear_fwd(X.q, W.q, Y, ws_lin)
            return
        ev_fork.record(main_stream)
        for o, st, ev in zip(ops, side, ev_join):
            st.wait_event(ev_fork)
            with torch.cuda.stream(st):
                o.prepare()
                ev.record(st)
        for ev in ev_join:
            main_stream.wait_event(ev)
        metis.fp4_linear_fwd(X.q, W.q, Y, ws_lin)
        if full:
            metis.fp4_linear_dgrad(G.q, W.q, dX, ws_lin)
            metis.fp4_linear_wgrad(G.q, X.q, dW, ws_lin)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones((1 << 28,), dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    n_split = sum(1 for o in ops if o.k)
    timers = {
        "gemm": metis.KernelTimer(metis.PROF_GEMM, args.steps * n_gemm),
        "broadcast": metis.KernelTimer(metis.PROF_BROADCAST, max(1, args.steps * n_split)),
        "residual_quant": metis.KernelTimer(metis.PROF_RESIDUAL_QUANT, max(1, args.steps * n_split)),
        "quantize": metis.KernelTimer(metis.PROF_QUANTIZE, max(1, args.steps)),
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

    useful_flops = 2.0 * L * K * N * n_gemm
    value = useful_flops / (ms_per_step * 1e-3) / 1e12

    def avg(name, count):
        d = timers[name].durations_ms(count)
        return sum(d) / len(d) if d else None

    gemm_ms = avg("gemm", args.steps * n_gemm)
    gemm_tflops = 2.0 * L * K * N / (gemm_ms * 1e-3) / 1e12
    roofline = {"kernel": "k_fp4_gemm_nt_pipe", "bound": "mfma", "achieved": round(gemm_tflops, 2),
                "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_MFMA_TFLOPS, 4),
                "traffic": None, "avg_launch_ms": round(gemm_ms, 4)}

    # per-call wall time of each entry point, measured after the timed region (5 repetitions)
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()                                      # kernels that no step has launched yet load on first use
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return round(e0.elapsed_time(e1) / 5, 4)

    phases = {}
    for name, o in (("W", W), ("X", X), ("G", G)):
        if o is None:
            continue
        if o.k:
            phases[f"decompose_{name}_ms"] = timed(lambda: metis.decompose(o.A, o.k, o.p, o.rho, o.seed, workspace=o.ws_dec,
                                                                        out=(o.U, o.S, o.V)))
            phases[f"split_quantize_{name}_ms"] = timed(lambda: metis.split_quantize(o.A, o.U, o.S, o.V, o.q,
                                                                                  workspace=o.ws_split))
        else:
            phases[f"quantize_{name}_ms"] = timed(lambda: metis.quantize(o.A, o.q.R, o.q.Rt))
    phases["linear_fwd_ms"] = timed(lambda: metis.fp4_linear_fwd(X.q, W.q, Y, ws_lin))
    if W.k:
        # gradients of W's factors from a dense dW (outside the timed step: an extra output of the backward pass)
        dWf = dW if full else torch.randn((N, K), dtype=torch.bfloat16, device="cuda")
        gU = torch.empty((N, W.k), dtype=torch.float32, device="cuda")
        gS = torch.empty((W.k, W.k), dtype=torch.float32, device="cuda")
        gV = torch.empty((K, W.k), dtype=torch.float32, device="cuda")
        ws_fg = torch.empty((metis.factor_grads_workspace_bytes(N, K, W.k),), dtype=torch.uint8, device="cuda")
        phases["factor_grads_W_ms"] = timed(lambda: metis.fp4_factor_grads(dWf, W.q, gU, gS, gV, ws_fg))
    if full:
        phases["linear_dgrad_ms"] = timed(lambda: metis.fp4_linear_dgrad(G.q, W.q, dX, ws_lin))
        phases["linear_wgrad_ms"] = timed(lambda: metis.fp4_linear_wgrad(G.q, X.q, dW, ws_lin))
    roofline["traffic"] = traffic_from_profile(args.workload)

    # The same product in the MXFP4 variant (block 32, power-of-two scales that the matrix instruction applies itself):
    # what the chip's FP4 rate gives when no expansion work is needed.  Outside the timed step and outside `value`.
    mx = None
    if K % 256 == 0:
        try:
            qx, qw = metis.MxTensor(L, K), metis.MxTensor(N, K)
            Ymx = torch.empty((L, N), dtype=torch.bfloat16, device="cuda")
            mx_q_ms = timed(lambda: (metis.quantize_mx(X.A, qx), metis.quantize_mx(W.A, qw)))
            mx_ms = timed(lambda: metis.mxfp4_gemm_nt(qx, qw, Ymx))
            mx_tf = 2.0 * L * K * N / (mx_ms * 1e-3) / 1e12
            mx = {"kernel": "k_mxfp4_gemm_nt", "quantize_both_ms": mx_q_ms, "gemm_ms": mx_ms, "achieved": round(mx_tf, 1),
                  "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s", "frac": round(mx_tf / PEAK_FP4_TFLOPS, 4)}
            del qx, qw, Ymx
        except Exception as e:                                     # an extra figure must never cost the main line
            mx = {"error": repr(e)[:200]}

    # Throughput with several independent steps in flight (different layers or micro-batches of a training
    # job): each slot has its own stream and its own outputs and workspaces, the inputs are shared.  A step's
    # decomposition is a chain of small single-workgroup kernels that leaves the chip idle; steps in other slots
    # fill it.  Reported beside `value`, which stays the one-step-at-a-time figure.
    pipelined = None
    depth = args.pipeline_depth
    if depth > 1 and not multi:
        try:
            pipelined = pipelined_throughput(args, torch, metis, oq, T, W, X, Y, ws_lin, p, full, depth, useful_flops)
        except Exception as e:                                     # an extra figure must never cost the main line
            pipelined = {"depth": depth, "error": repr(e)[:200]}

    passes = {}
    if n_split:
        bc_ms = avg("broadcast", args.steps * n_split)
        rq_ms = avg("residual_quant", args.steps * n_split)
        mn = sum(o.M * o.N for o in ops if o.k) / n_split
        orient = 2 if full else 1
        passes["broadcast"] = {"avg_ms": round(bc_ms, 4), "GB/s": round(2 * mn / bc_ms / 1e6, 1),
                               "frac_hbm": round(2 * mn / bc_ms / 1e6 / PEAK_HBM_GBS, 4)}
        rq_bytes = (2 + 0.5625 * orient) * mn
        passes["residual_quant"] = {"avg_ms": round(rq_ms, 4), "GB/s": round(rq_bytes / rq_ms / 1e6, 1),
                                    "frac_hbm": round(rq_bytes / rq_ms / 1e6 / PEAK_HBM_GBS, 4)}
    if not split_x:
        q_ms = avg("quantize", args.steps)
        qb = 2.5625 * L * K
        passes["quantize"] = {"avg_ms": round(q_ms, 4), "GB/s": round(qb / q_ms / 1e6, 1),
                              "frac_hbm": round(qb / q_ms / 1e6 / PEAK_HBM_GBS, 4)}
        # the stochastically rounded variant of the same pass (outside the timed step: the graded path rounds to nearest)
        sr_ms = timed(lambda: metis.quantize_sr(X.A, 1, X.q.R, None))
        passes["quantize_sr"] = {"avg_ms": round(sr_ms, 4), "GB/s": round(qb / sr_ms / 1e6, 1),
                                 "frac_hbm": round(qb / sr_ms / 1e6 / PEAK_HBM_GBS, 4)}
        metis.quantize(X.A, X.q.R, None)

    # The same HBM passes at the FFN activation shape (8192 x 14336, the largest matrix of a LLaMA-3-8B layer), one
    # operand at a time: on the 4096 x 4096 weight of the default workload a pass is a few microseconds of traffic
    # and mostly launch ramp, and on the three-operand workloads the figures above include the operands' contention.
    passes_ffn = None
    if not args.no_ffn_passes:
        try:
            passes_ffn = ffn_shape_passes(torch, metis, oq, k, p, prm["rho_x"])
        except Exception as e:                                     # an extra figure must never cost the main line
            passes_ffn = {"error": repr(e)[:200]}

    out = {
        "metric": "split-FP4 linear TFLOP/s + decompose/quantize GB/s (frac of roofline), 1 GPU",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4(e2m1)+e4m3 block scales, fp16 MFMA, fp32 accumulate", "data": "synthetic",
        "config": {"workload": {"c1": "config 1: tiny planted 256x512, X 128x512, k=8",
                                "c2": "config 2: LLaMA-3-8B attention projection W 4096x4096 (k=64,p=16) x X 8192x4096, "
                                      "decompose+split_quantize(W), quantize(X), fwd",
                                "c3": "config 3: FFN up W 14336x4096, X 8192x4096 both split, fwd",
                                "c4": "config 4: FFN down W 4096x14336, X 8192x14336, G 8192x4096, full W4A4G4 step"}[args.workload],
                   "L": L, "K": K, "N": N, "k": k, "p": p, "gemms_per_step": n_gemm, "setup_s": round(setup_s, 1)},
        "roofline": roofline,
        "pipelined": pipelined,
        "mxfp4_variant": mx,
        "passes": passes,
        "passes_ffn_shape": passes_ffn,
        "phases": phases,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, torch, T, c, prm, oq)
    print(json.dumps(out))


def ffn_shape_passes(torch, metis, oq, k, p, rho, reps=5):
    """Event-bracketed broadcast and residual + quantize kernels on one seeded 8192 x 14336 bf16 operand."""
    Mf, Nf = 8192, 14336
    gen = torch.Generator(device="cuda").manual_seed(20250904)
    Af = (torch.randn((Mf, Nf), generator=gen, device="cuda") * 0.05).to(torch.bfloat16)
    mn = Mf * Nf
    res = {"shape": [Mf, Nf], "k": k, "sample_rate": rho, "data": "seeded N(0, 0.05^2), timing only"}
    for want_t in (False, True):
        o = Operand(metis, torch, Af, k, p, rho, 11, want_t, oq)
        o.prepare()
        tb = metis.KernelTimer(metis.PROF_BROADCAST, reps)
        tr = metis.KernelTimer(metis.PROF_RESIDUAL_QUANT, reps)
        tb.__enter__()
        tr.__enter__()
        torch.cuda.synchronize()
        for _ in range(reps):
            o.prepare()
        torch.cuda.synchronize()
        tb.__exit__()
        tr.__exit__()
        bc, rq = tb.durations_ms(reps), tr.durations_ms(reps)
        bc_ms, rq_ms = sum(bc) / len(bc), sum(rq) / len(rq)
        if not want_t:
            res["broadcast"] = {"avg_ms": round(bc_ms, 4), "GB/s": round(2 * mn / bc_ms / 1e6, 1),
                                "frac_hbm": round(2 * mn / bc_ms / 1e6 / PEAK_HBM_GBS, 4)}
        rq_bytes = (2 + 0.5625 * (2 if want_t else 1)) * mn
        res["residual_quant_%d_orientation%s" % ((2, "s") if want_t else (1, ""))] = {
            "avg_ms": round(rq_ms, 4), "GB/s": round(rq_bytes / rq_ms / 1e6, 1),
            "frac_hbm": round(rq_bytes / rq_ms / 1e6 / PEAK_HBM_GBS, 4)}
        del o
    return res


def pipelined_throughput(args, torch, metis, oq, T, W, X, Y, ws_lin, p, full, depth, useful_flops):
    """Steps per second with `depth` independent steps in flight, each slot a HIP graph on its own stream."""
    slots = []
    for d in range(depth):
        Wd = Operand(metis, torch, T["W"], W.k, p, W.rho, W.seed, full, oq, share=W)
        Xd = Operand(metis, torch, T["X"], X.k, p, X.rho, X.seed, full, oq, share=X)
        slots.append((Wd, Xd, torch.empty_like(Y), torch.empty_like(ws_lin), torch.cuda.Stream()))

    def slot_step(sl):
        Wd, Xd, Yd, wsd, st = sl
        with torch.cuda.stream(st):
            Wd.prepare()
            Xd.prepare()
            metis.fp4_linear_fwd(Xd.q, Wd.q, Yd, wsd)

    for i in range(max(args.warmup, depth)):
        slot_step(slots[i % depth])
    torch.cuda.synchronize()
    # one HIP graph per slot: a step is ~35 launches, and with several steps in flight the host would
    # otherwise be the limit.  The library records kernels only (its buffers are cleared by fill kernels).
    graphs = []
    for sl in slots:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=sl[4]):
            sl[0].prepare()
            sl[1].prepare()
            metis.fp4_linear_fwd(sl[1].q, sl[0].q, sl[2], sl[3])
        graphs.append(g)
    torch.cuda.synchronize()

    def replay(i):
        with torch.cuda.stream(slots[i % depth][4]):
            graphs[i % depth].replay()

    for i in range(depth):
        slots[i][2].zero_()
        replay(i)
    torch.cuda.synchronize()
    t_p = time.perf_counter()
    for i in range(args.steps):
        replay(i)
    torch.cuda.synchronize()
    ms_p = (time.perf_counter() - t_p) * 1e3 / args.steps
    ref = Y.float()                                            # every slot reproduces the serial step's output
    same = all(((sl[2].float() - ref).abs().max() <= 1e-3 * ref.abs().max()).item() for sl in slots)
    pipelined = {"depth": depth, "ms_per_step": round(ms_p, 4),
                 "value": round(useful_flops / (ms_p * 1e-3) / 1e12, 3), "unit": "TFLOP/s",
                 "outputs_match_serial": bool(same)}
    del graphs, slots
    return pipelined


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


def cpu_baseline(np, torch, T, c, prm, oq):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import decompose as odec
    from oracle import linear as olin
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    k, p = prm["k"], prm["p"]
    Wn = T["W"].double().numpy()
    Xn = T["X"].double().numpy()
    rows = Xn.shape[0]
    # whole steps of the same workload, repeated until about ten seconds of oracle time have passed
    passes, t0, dt = 0, time.perf_counter(), 0.0
    while dt < 10.0 and passes < 64:
        U, S, V = odec.decompose(Wn, k, p, prm["rho_w"], 1)
        wq = olin.split_quantize(Wn, U, S, V, 2.0 ** -11, 2.0 ** -11, oq.tensor_scale_for(np.abs(Wn).max()), want_t=False)
        xq = olin.split_quantize(Xn, None, None, None, 1.0, 1.0, oq.tensor_scale_for(np.abs(Xn).max()), want_t=False)
        Yo = olin.linear_fwd(xq, wq)
        passes += 1
        dt = time.perf_counter() - t0
    flops = 2.0 * rows * Wn.shape[0] * Wn.shape[1] * passes
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": f"{passes} whole steps of the workload (decompose + split_quantize of W {Wn.shape[0]}x{Wn.shape[1]}, "
                      f"quantize + fwd of all {rows} rows of X); useful flops / oracle seconds"}


if __name__ == "__main__":
    main()
