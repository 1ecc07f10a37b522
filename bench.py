#!/usr/bin/env python3
"""Benchmark of the Float8 linear hot path on one MI355X.

A step = forward + backward of the seven Float8 linears of a Llama-3.1-8B
transformer block at M = 16384 tokens (the largest single-GPU configuration;
casts included), every tensor already resident in HBM.  Prints ONE JSON line:
whole-step TFLOP/s (6*M*K*N per linear), the roofline of the dominant kernel
(the fp8 GEMM, timed per launch with HIP events on the launch stream), the
amax+cast bandwidth, the shader clock of the timed steps, ceilings measured in
the same process (matrix pipes alone, device copy and read), one record per
other configuration (8B at M = 8192, 70B and 405B slices in their variants) in
`configs`, and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload KEY]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # dense bf16 MFMA peak of MI355X
PEAK_FP8_TFLOPS = 5000.0   # MI355X dense fp8 MFMA (published: 5.0 PFLOP/s)
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="default: llama8b_block (the seven 8B linears at M = 16384, the largest configuration) as the "
                         "headline, plus one record per other configuration in `configs`")
    ap.add_argument("--no-configs", action="store_true", help="default run: skip the other configurations")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured ceilings (MFMA-only loop, copy, read)")
    ap.add_argument("--variant", default=None, help="granularity:gradfmt, e.g. tensorwise:e4m3")
    ap.add_argument("--scaling", default="dynamic", choices=["dynamic", "delayed", "static"],
                    help="per-tensor scaling strategy (delayed/static: tensorwise only, single-pass casts)")
    ap.add_argument("--chain", action="store_true",
                    help="llama8b shapes only: feed wq's Y to wo and w1's Y to w2 (and the gradients back), "
                         "handing the amax from the producing GEMM's epilogue to the consumer's cast")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into a HIP graph once and time its replays")
    ap.add_argument("--recompute", nargs="?", const="full", default=None, choices=["full", "selective"],
                    help="llama8b_layer: activation checkpointing: run the forward again inside the backward (full), "
                         "or only its cheap bf16 operations, keeping the outputs of the products and of the attention (selective)")
    ap.add_argument("--keep-weights", action="store_true",
                    help="dynamic scaling: quantise the weights once before the timed steps and keep their codes "
                         "(micro-batches of one optimizer step); the default recasts them on every forward")
    ap.add_argument("--own-inputs", action="store_true",
                    help="llama8b_block: give wk, wv and w3 an input tensor and an input cast of their own instead of "
                         "sharing wq's and w1's")
    ap.add_argument("--transposed-copies", action="store_true",
                    help="tensorwise: also write every code tensor transposed (+1 B/elem) and run the backward as F8_NT "
                         "products on the copies, instead of reading the codes in place (F8_NN / F8_TN)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16-context", action="store_true",
                    help="skip timing torch.matmul in bf16 on the same shapes (context only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a device copy of known size (reference for the HBM byte counters)")
    ap.add_argument("--clock-study", action="store_true",
                    help="where the shader clock goes on the headline workload: the step, its GEMMs alone, its casts alone, "
                         "one product back to back and with idle gaps, the matrix pipes alone; one JSON line")
    ap.add_argument("--cpu-sample-rows", type=int, default=8192)
    return ap.parse_args()


class LinearState:
    """Device tensors of one linear of the workload."""

    def __init__(self, f8, w, li, inputs, rowwise, grad_fmt, scaling="dynamic", ws=None, transposed=False, x_owner=None):
        """x_owner: the LinearState of the linear whose input this one shares (it then reads that
        linear's X and the fp8 codes of it that the owner's forward leaves), or None."""
        import torch
        lin = w.linears[li]
        self.lin = lin
        self.X, self.W, self.dY = inputs
        self.x_owner = x_owner
        M, K, N = lin.M, lin.K, lin.N
        bf = dict(dtype=torch.bfloat16, device="cuda")
        self.Y = torch.empty((M, N), **bf)
        self.dX = torch.empty((M, K), **bf)
        self.dW = torch.empty((N, K), **bf)
        if x_owner is not None:
            self.X = x_owner.X
            self.saved = f8.Saved(M, K, N, rowwise, transposed=transposed, x=x_owner.saved.x)
        else:
            self.saved = f8.Saved(M, K, N, rowwise, transposed=transposed)
        self.desc = f8.linear_desc(M, K, N, rowwise, grad_fmt)
        self.state = f8.ScalingState(f8.DYNAMIC, 1) if x_owner is not None else None
        if scaling != "dynamic":
            # delayed: histories seeded with this batch's amax values (the first-step
            # initialisation); static: constant scales FMAX / amax of this batch
            self.state = f8.ScalingState(f8.DELAYED if scaling == "delayed" else f8.STATIC, 16)
            a = torch.empty(1, device="cuda")
            for key, t, fmt in (("x", self.X, f8.E4M3), ("w", self.W, f8.E4M3), ("dy", self.dY, grad_fmt)):
                f8.amax(t, f8.TENSORWISE, a, ws)
                f8.amax_history_push(getattr(self.state, "hist_" + key), a, fmt, getattr(self.state, "scale_" + key))


def shares_inputs(w, args, rowwise):
    """Whether the linears of `w` that read one activation share its cast in this run: the plain
    step under tensorwise scaling (the chained and kept-weight variants keep one input per linear)."""
    return bool(w.shared_x) and not rowwise and not args.own_inputs and not args.chain and not args.keep_weights


def make_states(f8, w, inputs, rowwise, grad_fmt, args, ws):
    states = []
    share = shares_inputs(w, args, rowwise)
    for li in range(len(w.linears)):
        own = w.x_owner(li) if share else li
        states.append(LinearState(f8, w, li, inputs[li], rowwise, grad_fmt, args.scaling, ws, args.transposed_copies,
                                  x_owner=states[own] if own != li else None))
    return states


def make_step(f8, torch, args, states, ws, rowwise):
    """The timed step of a linear workload: forward of every linear in model order, backward in reverse."""
    if args.chain:
        names = [s.lin.name for s in states]
        if args.scaling != "dynamic" or rowwise or names != ["wq", "wk", "wv", "wo", "w1", "w3", "w2"]:
            print("bench.py: --chain needs an 8B-shaped workload with dynamic tensorwise scaling", file=sys.stderr)
            sys.exit(2)
        chain_pairs = [(0, 3), (4, 6)]   # producer -> consumer: wq -> wo, w1 -> w2
        prod = {p: c for p, c in chain_pairs}
        cons = {c: p for p, c in chain_pairs}
        amax_y = {p: torch.empty(1, device="cuda") for p in prod}      # max |Y| of the producer
        amax_dx = {c: torch.empty(1, device="cuda") for c in cons}     # max |dX| of the consumer

        def step():
            for i, s in enumerate(states):
                if i in prod:
                    f8.linear_fwd_chained(s.desc, s.X, None, s.W, s.Y, amax_y[i], s.saved, ws)
                elif i in cons:
                    f8.linear_fwd_chained(s.desc, states[cons[i]].Y, amax_y[cons[i]], s.W, s.Y, None, s.saved, ws)
                else:
                    f8.linear_fwd(s.desc, s.X, s.W, s.Y, s.saved, ws)
            for i, s in reversed(list(enumerate(states))):
                if i in cons:
                    f8.linear_bwd_chained(s.desc, s.dY, None, s.saved, s.dX, amax_dx[i], s.dW, ws)
                elif i in prod:
                    f8.linear_bwd_chained(s.desc, states[prod[i]].dX, amax_dx[prod[i]], s.saved, s.dX, None, s.dW, ws)
                else:
                    f8.linear_bwd(s.desc, s.dY, s.saved, s.dX, s.dW, ws)
    elif args.scaling == "dynamic" and args.keep_weights:
        # gradient accumulation: the weights' fp8 codes are taken once (outside the timed steps)
        # and kept for the micro-batches that follow; NOT the headline accounting
        for s in states:
            f8.linear_fwd(s.desc, s.X, s.W, s.Y, s.saved, ws)

        def step():
            for s in states:
                f8.linear_fwd_wq(s.desc, s.X, s.Y, s.saved, ws)
            for s in reversed(states):
                f8.linear_bwd(s.desc, s.dY, s.saved, s.dX, s.dW, ws)
    elif args.scaling == "dynamic":
        def step():
            for s in states:                       # forward in model order
                if s.x_owner is None:
                    f8.linear_fwd(s.desc, s.X, s.W, s.Y, s.saved, ws)
                else:                              # the input's codes are the owner's: cast W, multiply
                    f8.linear_fwd_xq(s.desc, s.state, s.W, s.Y, s.saved, ws)
            for s in reversed(states):             # backward in reverse
                f8.linear_bwd(s.desc, s.dY, s.saved, s.dX, s.dW, ws)
    else:
        def step():
            for s in states:
                if s.x_owner is None:
                    f8.linear_fwd_scaled(s.desc, s.state, s.X, s.W, s.Y, s.saved, ws)
                else:
                    f8.linear_fwd_xq(s.desc, s.state, s.W, s.Y, s.saved, ws)
            for s in reversed(states):
                f8.linear_bwd_scaled(s.desc, s.state, s.dY, s.saved, s.dX, s.dW, ws)
    return step


def run_linear_workload(f8, wl, torch, args, w, gran, gfmt, steps, warmup, inputs=None):
    """Times `steps` steps of one linear workload in one variant and then its per-call legs.
    Returns (record, inputs): the record holds the step time, the whole-step rate, the GEMM and the
    cast legs; the device inputs are handed back so that another variant of the same workload can
    reuse them."""
    rowwise = gran == "rowwise"
    grad_fmt = f8.E5M2 if gfmt == "e5m2" else f8.E4M3
    dmax = max(max(l.M, l.K, l.N) for l in w.linears)
    ws = f8.new_workspace(dmax, dmax)
    if inputs is None:
        inputs = [tuple(t.cuda() for t in wl.make_linear_inputs(w, li)) for li in range(len(w.linears))]
    states = make_states(f8, w, inputs, rowwise, grad_fmt, args, ws)
    stream = torch.cuda.current_stream()   # the step and the per-call legs run on the current stream
    step = make_step(f8, torch, args, states, ws, rowwise)

    run_step = step
    if args.graph:
        # the library only enqueues kernels, so the whole step can be captured; the replay
        # issues the same kernels on the same buffers with one launch call
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            step()
        run_step = graph.replay
    for _ in range(warmup):
        run_step()
    clk = torch.zeros((2, 4 * f8.PROBE_CLOCK_SLOTS), dtype=torch.int64, device="cuda")
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    f8.probe_clock(clk[0], stream)
    marks[0].record(stream)
    for i in range(steps):
        run_step()
        marks[i + 1].record(stream)
    f8.probe_clock(clk[1], stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    ms_median = per_step[len(per_step) // 2]
    c = clk.cpu()
    # shader-clock cycles over 100 MHz ticks between the two sampling kernels that bracket the steps
    clock_ghz = f8.clock_ghz_between(c[0], c[1]) or 0.0
    flops_step = sum(s.lin.flops for s in states)
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---- per-call legs, HIP events on the launch stream ----------------------------------
    # An instrumented pass issues the step's own sequence of library calls (every tensor's
    # amax+cast and every GEMM, forward in model order, backward in reverse, through the same
    # C entry points the linear composes), each call between two events.  Same kernels, same
    # order and therefore the same cache state as in the timed steps.
    g = f8.ROWWISE if rowwise else f8.TENSORWISE
    reps = max(3, min(steps, 10))

    def cast_op(t, q, fmt):
        if args.scaling == "dynamic":   # the linear's own quantisation of one tensor
            return lambda: f8.quantise(t, g, fmt, q, ws, stream)
        if args.scaling == "delayed":
            return lambda: f8.cast_amax(t, q.scale, fmt, q.amax, q.q, q.q_t, ws, stream)
        return lambda: f8.cast(t, q.scale, f8.TENSORWISE, fmt, q.q, q.q_t, stream)

    ops = []  # (kind, linear index, call, flop or elements, name)
    for li, s in enumerate(states):
        M, K, N = s.lin.M, s.lin.K, s.lin.N
        sv = s.saved
        if s.x_owner is not None:       # X's codes are the owner's: only W is cast
            ops.append(("cast", li, cast_op(s.W, sv.w, f8.E4M3), s.W.numel(), "W"))
        elif args.scaling == "dynamic":   # the forward's own quantisation: X and W in one call
            ops.append(("cast", li, (lambda s=s, sv=sv: f8.linear_fwd_quantise(s.desc, s.X, s.W, sv, ws, stream)),
                        s.X.numel() + s.W.numel(), "X+W"))
        else:
            ops.append(("cast", li, cast_op(s.X, sv.x, f8.E4M3), s.X.numel(), "X"))
            ops.append(("cast", li, cast_op(s.W, sv.w, f8.E4M3), s.W.numel(), "W"))
        ops.append(("gemm", li, (lambda s=s, sv=sv, M=M, K=K, N=N: f8.gemm(
            f8.NT, M, N, K, sv.x.q, f8.E4M3, sv.w.q, f8.E4M3, sv.x.inv_scale, sv.w.inv_scale, g, s.Y, stream)),
            2 * M * K * N, "Y = X W^T"))
    for li, s in reversed(list(enumerate(states))):
        M, K, N = s.lin.M, s.lin.K, s.lin.N
        sv = s.saved
        w_is_t = sv.w.inv_scale_t if rowwise else sv.w.inv_scale
        dy_is_t = sv.dy.inv_scale_t if rowwise else sv.dy.inv_scale
        x_is_t = sv.x.inv_scale_t if rowwise else sv.x.inv_scale
        ops.append(("cast", li, cast_op(s.dY, sv.dy, grad_fmt), s.dY.numel(), "dY"))
        if sv.w.q_t is not None:   # rowwise, or --transposed-copies: F8_NT products on the transposed codes
            ops.append(("gemm", li, (lambda s=s, sv=sv, M=M, K=K, N=N, w_is_t=w_is_t: f8.gemm(
                f8.NT, M, K, N, sv.dy.q, grad_fmt, sv.w.q_t, f8.E4M3, sv.dy.inv_scale, w_is_t, g, s.dX, stream)),
                2 * M * K * N, "dX = dY W"))
            ops.append(("gemm", li, (lambda s=s, sv=sv, M=M, K=K, N=N, dy_is_t=dy_is_t, x_is_t=x_is_t: f8.gemm(
                f8.NT, N, K, M, sv.dy.q_t, grad_fmt, sv.x.q_t, f8.E4M3, dy_is_t, x_is_t, g, s.dW, stream, workspace=ws)),
                2 * M * K * N, "dW = dY^T X"))
        else:                      # the codes read in place: W and both of dY, X are k-major operands
            ops.append(("gemm", li, (lambda s=s, sv=sv, M=M, K=K, N=N: f8.gemm(
                f8.NN, M, K, N, sv.dy.q, grad_fmt, sv.w.q, f8.E4M3, sv.dy.inv_scale, sv.w.inv_scale, g, s.dX, stream)),
                2 * M * K * N, "dX = dY W"))
            ops.append(("gemm", li, (lambda s=s, sv=sv, M=M, K=K, N=N: f8.gemm(
                f8.TN, N, K, M, sv.dy.q, grad_fmt, sv.x.q, f8.E4M3, sv.dy.inv_scale, sv.x.inv_scale, g, s.dW, stream, workspace=ws)),
                2 * M * K * N, "dW = dY^T X"))

    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in ops]
           for _ in range(reps)]
    for _, _, fn, _, _ in ops:   # one untimed pass
        fn()
    for r in range(reps):
        for (a, b), (_, _, fn, _, _) in zip(evs[r], ops):
            a.record(stream)
            fn()
            b.record(stream)
    torch.cuda.synchronize()
    op_ms = [sum(evs[r][i][0].elapsed_time(evs[r][i][1]) for r in range(reps)) / reps for i in range(len(ops))]

    gemm_ms = sum(ms for ms, op in zip(op_ms, ops) if op[0] == "gemm")
    gemm_flops = sum(op[3] for op in ops if op[0] == "gemm")
    gemm_launches = sum(op[0] == "gemm" for op in ops)
    cast_ms = sum(ms for ms, op in zip(op_ms, ops) if op[0] == "cast")
    cast_elems = sum(op[3] for op in ops if op[0] == "cast")
    per_linear = []
    for li, s in enumerate(states):
        lg = sum(ms for ms, op in zip(op_ms, ops) if op[0] == "gemm" and op[1] == li)
        lc = sum(ms for ms, op in zip(op_ms, ops) if op[0] == "cast" and op[1] == li)
        per_linear.append({"name": s.lin.name, "M": s.lin.M, "K": s.lin.K, "N": s.lin.N,
                           "gemm_ms": round(lg, 4), "cast_ms": round(lc, 4),
                           "gemm_tflops": round(s.lin.flops / (lg * 1e-3) / 1e12, 1),
                           "tflops_by_product": {op[4]: round(op[3] / (ms * 1e-3) / 1e12, 1)
                                                 for ms, op in zip(op_ms, ops) if op[0] == "gemm" and op[1] == li},
                           "cast_us_by_tensor": {op[4]: round(ms * 1e3, 1)
                                                 for ms, op in zip(op_ms, ops) if op[0] == "cast" and op[1] == li}})
    by_product = {}
    for name in ("Y = X W^T", "dX = dY W", "dW = dY^T X"):
        fl = sum(op[3] for op in ops if op[0] == "gemm" and op[4] == name)
        t = sum(ms for ms, op in zip(op_ms, ops) if op[0] == "gemm" and op[4] == name)
        by_product[name] = round(fl / (t * 1e-3) / 1e12, 1)

    gemm_tflops = gemm_flops / (gemm_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "gemm_tile_kernel (fp8 MFMA 16x16x128; F8_NT forward, F8_NN and F8_TN backward)",
        "bound": "mfma",
        "achieved": round(gemm_tflops, 1),
        "peak": PEAK_FP8_TFLOPS,
        "unit": "TFLOP/s",
        "frac": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
        "traffic": None,
        "launches_per_step": gemm_launches,
        "tflops_by_product": by_product,
        "avg_launch_ms": round(gemm_ms / gemm_launches, 4),
        "flops_per_launch": gemm_flops // gemm_launches,
    }
    cast = None
    if cast_ms > 0:
        # dynamic tensorwise amax+cast: 2 B amax read + 2 B cast re-read + 1 B write per element
        # (with --transposed-copies a second code tensor is written: +1 B/elem moved, not counted).
        # delayed / static scaling: the scale is known beforehand, one pass: 2 B read + 1 B write.
        # rowwise: one amax pass yields the per-row and the per-column maxima (2 B), one cast pass
        # re-reads x (2 B) and writes the two differently scaled code sets (1 + 1 B): 6 B/elem.
        bpe = (6 if rowwise else 5) if args.scaling == "dynamic" else 3
        gbs = bpe * cast_elems / (cast_ms * 1e-3) / 1e9
        moved = bpe + (1 if (args.transposed_copies and not rowwise) else 0)
        cast = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_elem": bpe,
                "moved_gbs": round(moved * cast_elems / (cast_ms * 1e-3) / 1e9, 1),
                # the rate on the bytes a cast with a known scale would move (2 B read + 1 B written)
                "useful_bytes_gbs": round(3 * cast_elems / (cast_ms * 1e-3) / 1e9, 1),
                "ms_per_step": round(cast_ms, 4)}
    rec = {"workload": w.key, "ms_per_step": ms_per_step, "ms_per_step_median_of_events": ms_median,
           "tflops": tflops, "flops_step": flops_step, "shader_clock_ghz": clock_ghz,
           "roofline": roofline, "cast_roofline": cast, "per_linear": per_linear,
           "rowwise": rowwise, "grad_fmt": grad_fmt, "gran": gran, "gfmt": gfmt, "states": states, "reps": reps}
    return rec, inputs


def brief(rec):
    """One configuration's line of the `configs` object."""
    out = {"ms_per_step": round(rec["ms_per_step"], 4), "tflops": round(rec["tflops"], 1),
           "frac_of_fp8_peak": round(rec["tflops"] / PEAK_FP8_TFLOPS, 4),
           "gemm_kernels_tflops": rec["roofline"]["achieved"], "gemm_frac": rec["roofline"]["frac"],
           "shader_clock_ghz": round(rec["shader_clock_ghz"], 3),
           "variant": f"{rec['gran']}:{rec['gfmt']}"}
    if rec["cast_roofline"]:
        c = rec["cast_roofline"]
        out.update({"cast_gbs": c["achieved"], "cast_frac_of_hbm_peak": c["frac"], "cast_bytes_per_elem": c["bytes_per_elem"],
                    "cast_ms": c["ms_per_step"]})
    out["gemm_tflops_by_linear"] = {l["name"]: l["gemm_tflops"] for l in rec["per_linear"]}
    return out


# (config number of the benchmark spec, workload key, variants) of the `configs` object of the default run
ALL_CONFIGS = [(2, "llama8b", [("tensorwise", "e4m3")]),
               (3, "llama70b_tp8", [("tensorwise", "e4m3"), ("tensorwise", "e5m2")]),
               (4, "llama405b_tp8", [("tensorwise", "e4m3"), ("rowwise", "e4m3")])]
HEADLINE = "llama8b_block"   # config 5, the largest single-GPU configuration (21.4 TFLOP per step)


def measure_ceilings(f8, torch, codes):
    """What the chip delivers with nothing else in the way, measured in this process: the fp8 matrix
    pipes alone (constant operands, and the codes of a quantised tensor of this workload, whose
    switching activity is the GEMM's), a 1 GiB device copy and a 1 GiB device read."""
    stream = torch.cuda.current_stream()
    out = {}

    def time_ms(fn, reps):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    n = 1 << 24
    const = torch.full((n,), 0x38, dtype=torch.uint8, device="cuda")          # 1.0 everywhere
    flat = codes.reshape(-1)
    real = flat[: 1 << (flat.numel().bit_length() - 1)][:n].contiguous()       # a power of two of real codes
    iters = 2000
    for name, buf in (("constant_operands", const), ("workload_codes", real)):
        for shape, suffix in ((0, ""), (1, "_32x32x64")):
            fl = [0]

            def fn(buf=buf, shape=shape):
                fl[0] = f8.probe_mfma(buf, iters, ticks, sink, stream, shape=shape)
            ms = time_ms(fn, 3)
            t = ticks.cpu().tolist()
            n_mfma = iters * (64 if shape == 0 else 32)
            out["mfma_only_" + name + suffix] = {"tflops": round(fl[0] / (ms * 1e-3) / 1e12, 1),
                                                 "frac_of_nominal": round(fl[0] / (ms * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4),
                                                 "shader_clock_ghz": round(0.1 * t[0] / max(1, t[1]), 3),
                                                 "cycles_per_mfma": round(t[0] / n_mfma, 2)}
    gib = 1 << 30
    src = torch.empty(gib, dtype=torch.uint8, device="cuda")
    src.random_(0, 256)
    dst = torch.empty_like(src)
    sink32 = torch.zeros(1, dtype=torch.int32, device="cuda")
    ms = time_ms(lambda: f8.probe_copy(src, dst, stream), 5)
    out["copy_1GiB"] = {"gbs_read_plus_write": round(2 * gib / (ms * 1e-3) / 1e9, 1), "frac_of_nominal": round(2 * gib / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    ms = time_ms(lambda: f8.probe_read(src, sink32, stream), 5)
    out["read_1GiB"] = {"gbs": round(gib / (ms * 1e-3) / 1e9, 1), "frac_of_nominal": round(gib / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    out["what"] = ("f8_probe_mfma: one wave per SIMD, the 64 independent 16x16x128 fp8 MFMAs of a 128x128 wave tile per iteration "
                   "(the GEMM kernel's instruction; _32x32x64: the other fp8 instruction, 32 per iteration), operands in registers, "
                   "no LDS or memory traffic; f8_probe_copy / f8_probe_read: grid-stride 16-byte copy / read of 1 GiB")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_06511_amd import f8, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    f8.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    if args.copy_calibration:
        # 1 GiB read + 1 GiB written per launch, by the plain copy kernel of known size
        n = 1 << 30
        x = torch.ones(n, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(4):
            f8.probe_copy(x, y)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"kernel": "probe_copy_kernel", "bytes_read_per_launch": n,
                                                "bytes_written_per_launch": n, "launches": 4}}))
        return

    if args.workload == "attention":
        return attention_main(args)
    if args.clock_study:
        return clock_study(args)
    default_run = args.workload is None
    w = wl.WORKLOADS[args.workload or HEADLINE]
    if w.key == "llama8b_ffn":
        return ffn_main(args, w)
    if w.key == "llama8b_layer":
        return layer_main(args, w)
    gran, gfmt = (args.variant.split(":") if args.variant else w.variants[0])
    if args.scaling != "dynamic" and gran == "rowwise":
        print("bench.py: delayed and static scaling are per-tensor strategies; use a tensorwise variant",
              file=sys.stderr)
        sys.exit(2)

    rec, inputs = run_linear_workload(f8, wl, torch, args, w, gran, gfmt, args.steps, args.warmup)
    states, rowwise, grad_fmt = rec["states"], rec["rowwise"], rec["grad_fmt"]
    tflops, ms_per_step, flops_step = rec["tflops"], rec["ms_per_step"], rec["flops_step"]
    roofline = rec["roofline"]
    roofline["traffic"], roofline["traffic_source"] = committed_traffic()
    stream = torch.cuda.current_stream()

    def timed(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in ev) / reps  # ms

    out = {
        "metric": "Float8 linear fwd+bwd TFLOP/s (% FP8 MFMA peak) + amax/cast HBM GB/s",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8 (e4m3" + ("/e5m2 grads" if grad_fmt == f8.E5M2 else "") + ") x fp8 -> fp32 accumulate -> bf16",
        "data": "synthetic",
        "config": {"workload": f"{w.key}: " + ", ".join(f"{l.name}[M={l.M},K={l.K},N={l.N}]" for l in w.linears),
                   "scaling_granularity": gran, "scaling_strategy": args.scaling, "grad_format": gfmt, "chained": bool(args.chain), "hip_graph": bool(args.graph),
                   "shared_inputs": [[w.linears[i].name for i in g] for g in w.shared_x] if shares_inputs(w, args, rowwise) else [],
                   "weights_recast_every_step": not args.keep_weights, "transposed_code_copies": bool(args.transposed_copies or rowwise),
                   "flops_per_step": flops_step},
        "frac_of_fp8_peak": round(tflops / PEAK_FP8_TFLOPS, 4),
        "ms_per_step_median_of_events": round(rec["ms_per_step_median_of_events"], 4),
        "shader_clock_ghz_during_timed_steps": round(rec["shader_clock_ghz"], 3),
        "roofline": roofline,
        "cast_roofline": rec["cast_roofline"],
        "per_linear": rec["per_linear"],
    }

    if not args.no_ceilings:
        ceil = measure_ceilings(f8, torch, states[0].saved.x.q)
        out["ceilings"] = ceil
        m = ceil["mfma_only_workload_codes"]["tflops"]
        roofline["frac_of_measured_mfma_only_ceiling"] = round(roofline["achieved"] / m, 4)
        out["frac_of_measured_mfma_only_ceiling"] = round(tflops / m, 4)
        if rec["cast_roofline"]:
            rec["cast_roofline"]["frac_of_measured_copy_rate"] = round(
                rec["cast_roofline"]["achieved"] / ceil["copy_1GiB"]["gbs_read_plus_write"], 4)
        # the matrix pipes' rate at the clock the timed steps ran at
        at_clock = 256 * 4 * 2048 * rec["shader_clock_ghz"] * 1e9 / 1e12
        out["fp8_peak_at_measured_clock_tflops"] = round(at_clock, 1)
        roofline["frac_of_peak_at_measured_clock"] = round(roofline["achieved"] / at_clock, 4)
    if not args.no_bf16_context:
        out["bf16_matmul_context"] = bf16_context(states, timed, rec["reps"], flops_step)
        if not rowwise and grad_fmt == f8.E4M3:
            out["fp8_library_gemm_context"] = fp8_library_context(states, timed, rec["reps"], flops_step)
    if default_run and not args.no_configs:
        # every other configuration of the benchmark spec, each in the variants it names: fewer
        # steps, the same measurement
        configs = {f"config5 {w.key} {gran}:{gfmt}": brief(rec)}
        if shares_inputs(w, args, rowwise):
            # the same configuration with an input tensor and an input cast of its own for every linear
            # (seven X casts instead of four), for comparison
            import copy
            own_args = copy.copy(args)
            own_args.own_inputs = True
            del rec, states
            torch.cuda.empty_cache()
            orec, _ = run_linear_workload(f8, wl, torch, own_args, w, gran, gfmt, max(3, min(args.steps, 8)), 2, None)
            configs[f"config5 {w.key} {gran}:{gfmt}, every linear with its own input cast"] = brief(orec)
            del orec
            rec = states = None
        del rec, states, inputs
        torch.cuda.empty_cache()
        for num, key, variants in ALL_CONFIGS:
            cw, cin = wl.WORKLOADS[key], None
            for cg, cf in variants:
                crec, cin = run_linear_workload(f8, wl, torch, args, cw, cg, cf, max(3, min(args.steps, 8)), 2, cin)
                configs[f"config{num} {key} {cg}:{cf}"] = brief(crec)
                del crec
            del cin
            torch.cuda.empty_cache()
        out["configs"] = configs
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_rows, rowwise, grad_fmt, args.scaling)
    print(json.dumps(out))


def clock_study(args):
    """The same kernels in different company, each region bracketed by two shader-clock samples:
    how the clock (and with it the rate) depends on what else the chip is doing.  Rates are per
    region; `mfma_busy_frac` = TFLOP/s over what 1024 matrix pipes deliver at the region's clock."""
    import torch
    from paper_2410_06511_amd import f8, workloads as wl
    w = wl.WORKLOADS[HEADLINE]
    stream = torch.cuda.current_stream()
    dmax = max(max(l.M, l.K, l.N) for l in w.linears)
    ws = f8.new_workspace(dmax, dmax)
    inputs = [tuple(t.cuda() for t in wl.make_linear_inputs(w, li)) for li in range(len(w.linears))]
    args.scaling = "dynamic"
    dyn = make_states(f8, w, inputs, False, f8.E4M3, args, ws)
    step_dyn = make_step(f8, torch, args, dyn, ws, False)
    step_dyn()
    flops_step = sum(s.lin.flops for s in dyn)
    elems_step = sum((s.X.numel() if s.x_owner is None else 0) + s.W.numel() + s.dY.numel() for s in dyn)
    one = dyn[4]   # w1: Y = X W^T, 16384 x 14336 x 4096

    def gemms():
        for s in dyn:
            sv, l = s.saved, s.lin
            f8.gemm(f8.NT, l.M, l.N, l.K, sv.x.q, f8.E4M3, sv.w.q, f8.E4M3, sv.x.inv_scale, sv.w.inv_scale, f8.TENSORWISE, s.Y, stream)
        for s in reversed(dyn):
            sv, l = s.saved, s.lin
            f8.gemm(f8.NN, l.M, l.K, l.N, sv.dy.q, f8.E4M3, sv.w.q, f8.E4M3, sv.dy.inv_scale, sv.w.inv_scale, f8.TENSORWISE, s.dX, stream)
            f8.gemm(f8.TN, l.N, l.K, l.M, sv.dy.q, f8.E4M3, sv.x.q, f8.E4M3, sv.dy.inv_scale, sv.x.inv_scale, f8.TENSORWISE, s.dW, stream, workspace=ws)

    def casts():
        for s in dyn:
            if s.x_owner is None:
                f8.linear_fwd_quantise(s.desc, s.X, s.W, s.saved, ws, stream)
            else:
                f8.quantise(s.W, f8.TENSORWISE, f8.E4M3, s.saved.w, ws, stream)
        for s in reversed(dyn):
            f8.quantise(s.dY, f8.TENSORWISE, f8.E4M3, s.saved.dy, ws, stream)

    def one_product():
        sv, l = one.saved, one.lin
        f8.gemm(f8.NT, l.M, l.N, l.K, sv.x.q, f8.E4M3, sv.w.q, f8.E4M3, sv.x.inv_scale, sv.w.inv_scale, f8.TENSORWISE, one.Y, stream)

    def region(fn, reps, warm=3):
        for _ in range(warm):
            fn()
        clk = torch.zeros((2, 4 * f8.PROBE_CLOCK_SLOTS), dtype=torch.int64, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        f8.probe_clock(clk[0], stream)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        f8.probe_clock(clk[1], stream)
        torch.cuda.synchronize()
        c = clk.cpu()
        return e0.elapsed_time(e1) / reps, f8.clock_ghz_between(c[0], c[1]) or 0.0

    def rec(ms, ghz, flops=None, nbytes=None):
        r = {"ms": round(ms, 4), "shader_clock_ghz": round(ghz, 3)}
        if flops:
            tf = flops / (ms * 1e-3) / 1e12
            r.update({"tflops": round(tf, 1), "mfma_busy_frac": round(tf / (256 * 4 * 2048 * ghz * 1e-3), 4)})
        if nbytes:
            r["gbs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
        return r

    out = {"workload": w.key, "what": clock_study.__doc__.split("\n\n")[0].replace("\n    ", " ")}
    out["step_dynamic_scaling"] = rec(*region(step_dyn, args.steps), flops=flops_step)
    out["gemms_of_the_step_alone"] = rec(*region(gemms, args.steps), flops=flops_step)
    out["casts_of_the_step_alone"] = rec(*region(casts, args.steps), nbytes=5 * elems_step)
    one_flops = 2 * one.lin.M * one.lin.N * one.lin.K
    out["one_product_back_to_back"] = rec(*region(one_product, 40), flops=one_flops)
    out["one_product_back_to_back"]["product"] = f"w1 Y = X W^T, {one.lin.M} x {one.lin.N} x {one.lin.K}"
    # the same launch after 20 ms of idle, ten times: the chip starts each from its idle state
    gaps = []
    for _ in range(10):
        torch.cuda.synchronize()
        time.sleep(0.02)
        gaps.append(region(one_product, 1, warm=0))
    out["one_product_after_idle_gaps"] = rec(sum(g[0] for g in gaps) / len(gaps), sum(g[1] for g in gaps) / len(gaps), flops=one_flops)
    del dyn
    torch.cuda.empty_cache()
    # delayed scaling: every cast is one pass (3 instead of 5 bytes per element), the GEMMs are the same
    args.scaling = "delayed"
    dly = make_states(f8, w, inputs, False, f8.E4M3, args, ws)
    step_dly = make_step(f8, torch, args, dly, ws, False)
    out["step_delayed_scaling"] = rec(*region(step_dly, args.steps), flops=flops_step)
    ceil = measure_ceilings(f8, torch, dly[0].saved.x.q)
    for k in ("mfma_only_constant_operands", "mfma_only_workload_codes", "mfma_only_workload_codes_32x32x64"):
        out[k] = ceil[k]
    print(json.dumps(out))


def ffn_main(args, w):
    """The chained feed-forward block: stacked w1|w3 linear, silu(a) * b glue with the amax of
    its output taken in the same pass, w2 linear; then the backward chain.  FLOPs counted are
    the linears' (6 M K N each); the glue's time is inside the step."""
    import torch
    from paper_2410_06511_amd import f8, workloads as wl
    l13, l2 = w.linears
    M, D, H = l13.M, l13.K, l2.K
    assert l13.N == 2 * H and l2.N == D
    X, W13, _ = wl.make_linear_inputs(w, 0)
    _, W2, dY = wl.make_linear_inputs(w, 1)
    X, W13, W2, dY = X.cuda(), W13.cuda(), W2.cuda(), dY.cuda()
    bf = dict(dtype=torch.bfloat16, device="cuda")
    d13, d2 = f8.linear_desc(M, D, 2 * H), f8.linear_desc(M, H, D)
    s13, s2 = f8.Saved(M, D, 2 * H), f8.Saved(M, H, D)
    ws = f8.new_workspace(max(M, D, 2 * H), max(M, D, 2 * H))
    AB, Hh, Y = torch.empty((M, 2 * H), **bf), torch.empty((M, H), **bf), torch.empty((M, D), **bf)
    dH, dAB, dX = torch.empty((M, H), **bf), torch.empty((M, 2 * H), **bf), torch.empty((M, D), **bf)
    dW13, dW2 = torch.empty((2 * H, D), **bf), torch.empty((D, H), **bf)
    a_h, a_dab, a_xn = (torch.empty(1, device="cuda") for _ in range(3))
    Xn, gw = torch.empty((M, D), **bf), torch.ones(D, **bf)
    stream = torch.cuda.current_stream()

    delayed = args.scaling == "delayed"
    if args.scaling == "static":
        print("bench.py: the feed-forward chain runs with dynamic or delayed scaling", file=sys.stderr)
        sys.exit(2)
    if delayed:
        # delayed scaling: every scale is known beforehand, so the glue is fused into the casts of
        # w2's input and of w13's output gradient (h and dAB are never written) and no amax has
        # to be handed over
        st13, st2 = f8.ScalingState(f8.DELAYED, 16), f8.ScalingState(f8.DELAYED, 16)
        calls = [
            ("rmsnorm", lambda: f8.rmsnorm(X, gw, 1e-5, Xn, None, None, None, stream), 0, 4 * M * D),
            ("linear w13 fwd", lambda: f8.linear_fwd_scaled(d13, st13, Xn, W13, AB, s13, ws, stream), 2 * M * D * 2 * H, 0),
            ("silu_mul fused into the cast of h", lambda: f8.silu_mul_quantise_delayed(AB, f8.E4M3, st2.hist_x, st2.scale_x, s2.x, ws, stream), 0, 6 * M * H),
            ("linear w2 fwd (input already quantised)", lambda: f8.linear_fwd_xq(d2, st2, W2, Y, s2, ws, stream), 2 * M * H * D, 0),
            ("linear w2 bwd", lambda: f8.linear_bwd_scaled(d2, st2, dY, s2, dH, dW2, ws, stream), 4 * M * H * D, 0),
            ("silu_mul_bwd fused into the cast of dAB", lambda: f8.silu_mul_bwd_quantise_delayed(AB, dH, f8.E4M3, st13.hist_dy, st13.scale_dy, s13.dy, ws, stream), 0, 10 * M * H),
            ("linear w13 bwd (gradient already quantised)", lambda: f8.linear_bwd_dyq(d13, s13, dX, dW13, stream), 4 * M * D * 2 * H, 0),
        ]
        # seed the histories with one dynamic pass (the first-step initialisation)
        a = torch.empty(1, device="cuda")
        f8.rmsnorm(X, gw, 1e-5, Xn, None, None, None, stream)
        f8.linear_fwd_chained(d13, Xn, None, W13, AB, None, s13, ws, stream)
        f8.silu_mul(AB, Hh, a_h, ws, stream)
        f8.linear_fwd_chained(d2, Hh, a_h, W2, Y, None, s2, ws, stream)
        f8.linear_bwd_chained(d2, dY, None, s2, dH, None, dW2, ws, stream)
        f8.silu_mul_bwd(AB, dH, dAB, a_dab, ws, stream)
        for stt, key, src, fmt in ((st13, "x", s13.x.amax, f8.E4M3), (st13, "w", s13.w.amax, f8.E4M3), (st13, "dy", a_dab, f8.E4M3),
                                   (st2, "x", a_h, f8.E4M3), (st2, "w", s2.w.amax, f8.E4M3), (st2, "dy", s2.dy.amax, f8.E4M3)):
            f8.amax_history_push(getattr(stt, "hist_" + key), src, fmt, getattr(stt, "scale_" + key), None, stream)
    # (name, call, linear flop, algorithmic bytes of a glue kernel)
    calls = calls if delayed else [
        ("rmsnorm", lambda: f8.rmsnorm(X, gw, 1e-5, Xn, None, a_xn, ws, stream), 0, 4 * M * D),
        ("linear w13 fwd", lambda: f8.linear_fwd_chained(d13, Xn, a_xn, W13, AB, None, s13, ws, stream), 2 * M * D * 2 * H, 0),
        ("silu_mul", lambda: f8.silu_mul(AB, Hh, a_h, ws, stream), 0, 6 * M * H),
        ("linear w2 fwd", lambda: f8.linear_fwd_chained(d2, Hh, a_h, W2, Y, None, s2, ws, stream), 2 * M * H * D, 0),
        ("linear w2 bwd", lambda: f8.linear_bwd_chained(d2, dY, None, s2, dH, None, dW2, ws, stream), 4 * M * H * D, 0),
        ("silu_mul_bwd", lambda: f8.silu_mul_bwd(AB, dH, dAB, a_dab, ws, stream), 0, 10 * M * H),
        ("linear w13 bwd", lambda: f8.linear_bwd_chained(d13, dAB, a_dab, s13, dX, None, dW13, ws, stream), 4 * M * D * 2 * H, 0),
    ]

    def step():
        for _, fn, _, _ in calls:
            fn()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    flops_step = sum(l.flops for l in w.linears)
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    reps = max(3, min(args.steps, 10))
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls] for _ in range(reps)]
    for r in range(reps):
        for (a, b), (_, fn, _, _) in zip(evs[r], calls):
            a.record(stream)
            fn()
            b.record(stream)
    torch.cuda.synchronize()
    legs = []
    for i, (name, _, fl, by) in enumerate(calls):
        ms = sum(evs[r][i][0].elapsed_time(evs[r][i][1]) for r in range(reps)) / reps
        leg = {"call": name, "ms": round(ms, 4)}
        if fl:
            leg["tflops_incl_casts"] = round(fl / (ms * 1e-3) / 1e12, 1)
        if by:
            leg["gbs"] = round(by / (ms * 1e-3) / 1e9, 1)
            leg["bytes_per_elem"] = by // (M * D if name == "rmsnorm" else M * H)
            if name.startswith("silu_mul fused"):
                leg["note"] = "reads [a | b] (4 B), writes the codes of h (1 B; 2 B with a transposed copy); replaces silu_mul (6 B) + the cast of h (4 B)"
            if name.startswith("silu_mul_bwd fused"):
                leg["note"] = "reads [a | b] and dh (6 B), writes the codes of dAB (2 B; 4 B with a transposed copy); replaces silu_mul_bwd (10 B) + the cast of dAB (8 B)"
        legs.append(leg)
    glue_ms = sum(l["ms"] for l in legs if "gbs" in l)
    glue_bytes = sum(by for _, _, _, by in calls)
    out = {
        "metric": "Float8 linear fwd+bwd TFLOP/s (% FP8 MFMA peak) + amax/cast HBM GB/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8 (e4m3) x fp8 -> fp32 accumulate -> bf16", "data": "synthetic",
        "config": {"workload": f"{w.key}: chained feed-forward block, M={M}, hidden {D}, FFN {H}: "
                               "rmsnorm -> w1|w3 stacked [N=2*FFN] -> silu(a)*b -> w2, and the backward of the three linear stages",
                   "scaling_granularity": "tensorwise", "scaling_strategy": args.scaling, "grad_format": "e4m3",
                   "chained": True, "flops_per_step": flops_step},
        "frac_of_fp8_peak": round(tflops / PEAK_FP8_TFLOPS, 4),
        "roofline": {"kernel": "rmsnorm_kernel + silu_mul_kernel + silu_mul_bwd_kernel (the glue; the GEMM figures "
                               "are those of the linear workloads)", "bound": "hbm",
                     "achieved": round(glue_bytes / (glue_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(glue_bytes / (glue_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None},
        "legs": legs,
    }
    print(json.dumps(out))


def attention_main(args):
    """The block's causal grouped-query attention alone, forward and backward, at the Llama 3.1 8B
    shape (one sequence of 8192 tokens, 32 query and 8 key/value heads of 128) on seeded inputs;
    also the program that the attention kernels' counter summaries under profiles/ are collected
    on.  `value` is the attention's own rate on causal FLOPs (4 S^2 Hq hd / 2 forward, 2.5 times that
    backward), against the bf16 matrix peak."""
    import torch
    from paper_2410_06511_amd import f8
    B, S, Hq, Hkv, HD = 1, 8192, 32, 8, 128
    M = B * S
    g = torch.Generator("cpu")
    g.manual_seed(8192)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    qkv = torch.randn((M, (Hq + 2 * Hkv) * HD), generator=g).bfloat16().cuda()
    do = (torch.randn((M, Hq * HD), generator=g) * 0.01).bfloat16().cuda()
    q, k, v = qkv[:, :Hq * HD], qkv[:, Hq * HD:(Hq + Hkv) * HD], qkv[:, (Hq + Hkv) * HD:]
    vt, o = torch.empty((Hkv * HD, M), **bf), torch.empty((M, Hq * HD), **bf)
    qt, kt, dot = torch.empty((Hq * HD, M), **bf), torch.empty((Hkv * HD, M), **bf), torch.empty((Hq * HD, M), **bf)
    lse, delta = torch.empty((Hq, M), device="cuda"), torch.empty((Hq, M), device="cuda")
    dqkv = torch.zeros((M, (Hq + 2 * Hkv) * HD), **bf)
    dq, dk, dv = dqkv[:, :Hq * HD], dqkv[:, Hq * HD:(Hq + Hkv) * HD], dqkv[:, (Hq + Hkv) * HD:]
    ws = torch.empty(f8.sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, HD), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    for src, dst in ((v, vt), (q, qt), (k, kt), (do, dot)):
        f8.transpose_bf16(src, dst)
    fwd = lambda: f8.sdpa_fwd(q, k, vt, B, S, Hq, Hkv, HD, o, lse)
    bwd = lambda: f8.sdpa_bwd(q, qt, k, kt, v, o, do, dot, lse, B, S, Hq, Hkv, HD, dq, dk, dv, delta, ws)
    for _ in range(args.warmup):
        fwd(), bwd()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record(stream)
    for i in range(args.steps):
        fwd()
        ev[2 * i + 1].record(stream)
        bwd()
        ev[2 * i + 2].record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    f_ms = sum(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(args.steps)) / args.steps
    b_ms = sum(ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(args.steps)) / args.steps
    f_fl = 4 * B * S * S * Hq * HD // 2
    fl = f_fl + 5 * f_fl // 2
    tf = fl / (ms_per_step * 1e-3) / 1e12
    print(json.dumps({
        "metric": "causal attention fwd+bwd TFLOP/s (bf16 MFMA)", "value": round(tf, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16 x bf16 -> fp32", "data": "synthetic",
        "config": {"workload": f"attention: causal GQA, {B} x {S} tokens, {Hq} query / {Hkv} key-value heads of {HD}"},
        "forward_ms": round(f_ms, 4), "backward_ms": round(b_ms, 4),
        "roofline": {"kernel": "sdpa_fwd_kernel + sdpa_bwd_dq_kernel + sdpa_bwd_dkv_kernel", "bound": "mfma", "achieved": round(tf, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": None}}))


def layer_main(args, w):
    """One whole transformer block, forward and backward: the Float8 linears chained through the
    bf16 operations between them.  `value` counts the linears' FLOPs only (6 M K N each), as for
    every other workload; the attention's FLOPs and every bf16 stage's time are inside the step
    and itemised in `legs`."""
    import torch
    from paper_2410_06511_amd import workloads as wl
    from paper_2410_06511_amd.block import TransformerBlock
    if args.scaling == "static":
        print("bench.py: the transformer block runs with dynamic or delayed scaling", file=sys.stderr)
        sys.exit(2)
    sh = wl.LAYER_SHAPE[w.key]
    B, S, Hq, Hkv, hd, D, H = (sh[k] for k in ("B", "S", "Hq", "Hkv", "hd", "D", "H"))
    M = B * S
    g = torch.Generator("cpu")
    g.manual_seed(wl.seed_for(w.config_index, 0, "x"))
    x = wl.randn_bf16((M, D), 1.0, 0, generator=g).cuda()
    dout = wl.randn_bf16((M, D), 1e-3, 0, generator=g).cuda()
    # weights: N(0, 0.02) as in the other workloads, except that wq, wk are larger so that the
    # attention is not uniform (scores of order one)
    weights = {"g1": torch.ones(D, dtype=torch.bfloat16, device="cuda"), "g2": torch.ones(D, dtype=torch.bfloat16, device="cuda"),
               "Wqkv": wl.randn_bf16(((Hq + 2 * Hkv) * hd, D), 0.05, 0, generator=g).cuda(),
               "Wo": wl.randn_bf16((D, D), 0.02, 0, generator=g).cuda(),
               "W13": wl.randn_bf16((2 * H, D), 0.02, 0, generator=g).cuda(),
               "W2": wl.randn_bf16((D, H), 0.02, 0, generator=g).cuda()}
    blk = TransformerBlock(B, S, D, H, Hq, Hkv, hd, scaling=args.scaling)
    stream = torch.cuda.current_stream()

    def step():
        blk.forward(x, weights, stream)
        blk.backward(x, weights, dout, stream, recompute={"full": True, "selective": "selective", None: False}[args.recompute])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    flops_step = sum(l.flops for l in w.linears)
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    calls = blk.forward_stages(x, weights, stream) + blk.backward_stages(x, weights, dout, stream)
    reps = max(3, min(args.steps, 10))
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls] for _ in range(reps)]
    for r in range(reps):
        for (a, b), (_, fn, _, _) in zip(evs[r], calls):
            a.record(stream)
            fn()
            b.record(stream)
    torch.cuda.synchronize()
    legs, lin_ms, att_ms, att_flops, glue_ms, glue_bytes = [], 0.0, 0.0, 0, 0.0, 0
    for i, (name, _, fl, by) in enumerate(calls):
        ms = sum(evs[r][i][0].elapsed_time(evs[r][i][1]) for r in range(reps)) / reps
        leg = {"call": name, "ms": round(ms, 4)}
        if fl:
            leg["tflops"] = round(fl / (ms * 1e-3) / 1e12, 1)
            if name.startswith("attention"):
                att_ms, att_flops = att_ms + ms, att_flops + fl
            else:
                lin_ms += ms
        if by:
            leg["gbs"] = round(by / (ms * 1e-3) / 1e9, 1)
            glue_ms, glue_bytes = glue_ms + ms, glue_bytes + by
        legs.append(leg)
    att_tflops = att_flops / (att_ms * 1e-3) / 1e12
    context = None
    if not args.no_bf16_context:
        # Context, not part of the path: the library attention (torch's scaled_dot_product_attention,
        # forward and backward through autograd) on tensors of the same shape.
        F = torch.nn.functional
        qh = torch.randn((B, Hq, S, hd), dtype=torch.bfloat16, device="cuda", requires_grad=True)
        kh = torch.randn((B, Hkv, S, hd), dtype=torch.bfloat16, device="cuda", requires_grad=True)
        vh = torch.randn((B, Hkv, S, hd), dtype=torch.bfloat16, device="cuda", requires_grad=True)
        go = torch.randn((B, Hq, S, hd), dtype=torch.bfloat16, device="cuda") * 1e-2
        try:
            def lib_attention():
                o = F.scaled_dot_product_attention(qh, kh, vh, is_causal=True, enable_gqa=True)
                o.backward(go)
                qh.grad = kh.grad = vh.grad = None
            for _ in range(2):
                lib_attention()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(5):
                lib_attention()
            e1.record(stream)
            torch.cuda.synchronize()
            context = {"ms_fwd_bwd": round(e0.elapsed_time(e1) / 5, 4),
                       "what": "torch.nn.functional.scaled_dot_product_attention (is_causal, enable_gqa) forward + autograd backward, same shape"}
        except Exception as exc:  # the library path is context only
            context = {"error": str(exc)[:200]}
    out = {
        "metric": "Float8 linear fwd+bwd TFLOP/s (% FP8 MFMA peak) + amax/cast HBM GB/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8 (e4m3) x fp8 -> fp32 accumulate -> bf16 (linears); bf16 x bf16 -> fp32 (attention)", "data": "synthetic",
        "config": {"workload": f"{w.key}: one Llama 3.1 8B transformer block, {B} x {S} tokens, hidden {D}, FFN {H}, "
                               f"{Hq} query / {Hkv} key-value heads of {hd}: rmsnorm -> wq|wk|wv -> rope -> causal attention -> wo -> "
                               "+x -> rmsnorm -> w1|w3 -> silu(a)*b -> w2 -> +h, and the backward of every stage",
                   "scaling_granularity": "tensorwise", "scaling_strategy": args.scaling, "grad_format": "e4m3",
                   "chained": True, "recompute_in_backward": args.recompute or "none", "flops_per_step": flops_step,
                   "attention_flops_per_step_not_counted": att_flops},
        "frac_of_fp8_peak": round(tflops / PEAK_FP8_TFLOPS, 4),
        "linears_ms": round(lin_ms, 4), "attention_ms": round(att_ms, 4), "bf16_glue_ms": round(glue_ms, 4),
        "roofline": {"kernel": "sdpa_fwd_kernel + sdpa_bwd_dq_kernel + sdpa_bwd_dkv_kernel (the attention, which is what this "
                               "workload adds; the GEMM figures are those of the linear workloads); causal FLOPs: "
                               "4 S^2 Hq hd / 2 forward, 2.5 times that backward (recomputed scores not counted)",
                     "bound": "mfma", "achieved": round(att_tflops, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(att_tflops / PEAK_BF16_TFLOPS, 4), "traffic": None},
        "glue_gbs": round(glue_bytes / (glue_ms * 1e-3) / 1e9, 1),
        "library_attention_context": context,
        "legs": legs,
    }
    print(json.dumps(out))


def bf16_context(states, timed, reps, flops_step):
    """Context, not part of the path: the three matrix products of every linear as plain bf16
    torch.matmul calls (the library GEMM that the Float8 linear replaces), no casts."""
    import torch
    total = 0.0
    for s in states:
        fns = [lambda: torch.matmul(s.X, s.W.t(), out=s.Y),
               lambda: torch.matmul(s.dY, s.W, out=s.dX),
               lambda: torch.matmul(s.dY.t(), s.X, out=s.dW)]
        for fn in fns:
            fn()
            total += timed(fn, reps)
    return {"ms_per_step": round(total, 4), "tflops": round(flops_step / (total * 1e-3) / 1e12, 1),
            "what": f"torch.matmul bf16 (hipBLASLt), the same {3 * len(states)} products, no casts"}


TRAFFIC_SUMMARY = "gemm_cast_llama8b_block_hbm_traffic.md"


def fp8_library_context(states, timed, reps, flops_step):
    """Context, not part of the path: the vendor library's fp8 GEMM (torch._scaled_mm, which goes
    to hipBLASLt) on the same products, fed the codes this library produced, with the operands
    that call wants transposed copied beforehand (untimed).  E4M3 tensorwise only."""
    import torch
    try:
        total = 0.0
        by_product = {"Y = X W^T": [0.0, 0], "dX = dY W": [0.0, 0], "dW = dY^T X": [0.0, 0]}
        for s in states:
            sv = s.saved
            x8, w8, dy8 = (t.view(torch.float8_e4m3fn) for t in (sv.x.q, sv.w.q, sv.dy.q))
            w8t, dy8t, x8t = w8.t().contiguous(), dy8.t().contiguous(), x8.t().contiguous()
            isx, isw, isdy = sv.x.inv_scale.reshape(()), sv.w.inv_scale.reshape(()), sv.dy.inv_scale.reshape(())
            fns = [lambda: torch._scaled_mm(x8, w8.t(), isx, isw, out_dtype=torch.bfloat16),          # Y  = X W^T
                   lambda: torch._scaled_mm(dy8, w8t.t(), isdy, isw, out_dtype=torch.bfloat16),       # dX = dY W
                   lambda: torch._scaled_mm(dy8t, x8t.t(), isdy, isx, out_dtype=torch.bfloat16)]      # dW = dY^T X
            for fn, name in zip(fns, by_product):
                fn()
                ms = timed(fn, reps)
                total += ms
                by_product[name][0] += ms
                by_product[name][1] += 2 * s.lin.M * s.lin.K * s.lin.N
        return {"ms_per_step": round(total, 4), "tflops": round(flops_step / (total * 1e-3) / 1e12, 1),
                "tflops_by_product": {k: round(fl / (ms * 1e-3) / 1e12, 1) for k, (ms, fl) in by_product.items()},
                "what": f"torch._scaled_mm fp8 e4m3 (hipBLASLt), the same {3 * len(states)} products on this library's codes, "
                        "operands pre-transposed as that call wants them, no casts"}
    except Exception as exc:   # context only
        return {"error": str(exc)[:300]}


def committed_traffic():
    """(bytes per GEMM launch between L2 and the fabric / HBM, where the figure comes from): taken
    from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by a copy of known size)
    summarised under profiles/, which also names the source revision it was measured at; (None,
    reason) if that summary is absent.  Measured on the default workload, not in this process."""
    path = os.path.join(ROOT, "profiles", TRAFFIC_SUMMARY)
    val, rev = None, "unknown revision"
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_gemm_launch:"):
                val = int(ln.split(":")[1])
            if ln.startswith("measured_at_revision:"):
                rev = ln.split(":", 1)[1].strip()
    except OSError:
        return None, "profiles/" + TRAFFIC_SUMMARY + " is absent"
    return val, f"profiles/{TRAFFIC_SUMMARY}, kernels as of {rev}"


def cpu_baseline(w, rows, rowwise, grad_fmt, scaling="dynamic"):
    """The oracle as it stands, on the host cores, on a bounded sample: the narrowest linear
    of the workload restricted to its first `rows` tokens, forward + backward, casts included."""
    import oracle as o
    from paper_2410_06511_amd import workloads as wl
    li = min(range(len(w.linears)), key=lambda i: w.linears[i].K * w.linears[i].N)
    lin = w.linears[li]
    rows = min(rows, lin.M)
    X, W, dY = wl.make_linear_inputs(w, li, M=rows)
    xb, wb, dyb = wl.bits(X), wl.bits(W), wl.bits(dY)
    if scaling == "dynamic":
        t0 = time.perf_counter()
        _, xq, wq = o.linear_fwd(xb, wb, rowwise)
        o.linear_bwd(dyb, xq, wq, rowwise, grad_fmt)
        dt = time.perf_counter() - t0
    else:
        st = o.ScalingState(o.DELAYED if scaling == "delayed" else o.STATIC, 16)
        for key, t, fmt in (("x", xb, o.E4M3), ("w", wb, o.E4M3), ("dy", dyb, grad_fmt)):
            st.scale[key], _ = o.history_push(st.hist[key], o.amax(t)[0], fmt)
        t0 = time.perf_counter()
        _, xq, wq = o.linear_fwd_scaled(xb, wb, st)
        o.linear_bwd_scaled(dyb, xq, wq, st, grad_fmt)
        dt = time.perf_counter() - t0
    fl = 6 * rows * lin.K * lin.N
    value = fl / dt / 1e12
    # amax -> scale -> cast of that linear's whole X (O(elements), so timed at full size)
    Xf = wl.bits(wl.make_linear_inputs(w, li)[0])
    t0 = time.perf_counter()
    o.amax_cast(Xf, o.ROWWISE if rowwise else o.TENSORWISE, o.E4M3)
    dtc = time.perf_counter() - t0
    step_flops = sum(l.flops for l in w.linears)
    return {"value": round(value, 6), "unit": "TFLOP/s", "cores": o.num_threads(), "kind": "oracle",
            "sample": f"{w.key}/{lin.name} (K={lin.K}, N={lin.N}) first {rows} of {lin.M} tokens, fwd+bwd with casts",
            "seconds": round(dt, 2),
            "amax_cast": {"gbs": round(5 * Xf.size / dtc / 1e9, 3), "bytes_per_elem": 5, "seconds": round(dtc, 3),
                          "sample": f"{w.key}/{lin.name} X [{Xf.shape[0]}, {Xf.shape[1]}], whole tensor"},
            "extrapolated": {"seconds_per_step_of_the_whole_workload": round(step_flops / (value * 1e12), 1),
                             "how": "the workload's FLOPs per step at the sample's rate (the oracle's time is linear in M K N); not measured"}}


if __name__ == "__main__":
    main()
