#!/usr/bin/env python3
"""Benchmark of the per-tensor FP8 linear hot path (fwd + bwd, fused TWEO penalty) on one MI355X.

A step = one pass over every linear layer of the workload's Transformer block (all forwards, then
the backwards in reverse order, as a training step runs them), each from its
bf16 operands: amax(X), amax(W), E4M3 casts (+ transposes), FP8 forward GEMM with the penalty
epilogue, amax(dY), cast of dY, dgrad GEMM, wgrad GEMM.  Inputs are synthetic (seeded), resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama|gpt2|vit|single]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOADS = {"single": 0, "gpt2": 1, "vit": 2, "llama": 3}
PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "fp8_gemm_llama_block_pmc_traffic.txt")
FP8_PEAK_TFLOPS = 5000.0   # MI355X dense FP8 MFMA
INT8_PEAK_TOPS = 5000.0
HBM_PEAK_GBS = 8000.0
PEN = (3.0, 1e-6, 4)       # tau, eps, p of the paper's experiments


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Device buffers of one linear layer (all allocated up front; the library allocates nothing)."""

    def __init__(self, tw, torch, synth, cfg, gi, dev):
        g = synth.CONFIGS[cfg]["gemms"][gi]
        self.name, self.M, self.K, self.N = g.name, g.M, g.K, g.N
        M, K, N = g.M, g.K, g.N
        x, w, dy = synth.fp8_linear_inputs(cfg, gi)
        self.host = (x, w, dy)
        up = lambda b: torch.from_numpy(b.view("int16")).to(dev).view(torch.bfloat16)
        self.x, self.w, self.dy = up(x), up(w), up(dy)
        u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=dev)
        bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=dev)
        self.xq, self.xqT, self.wq, self.wqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N)
        self.dyq, self.dyqT = u8(M, N), u8(N, M)
        self.y, self.dx, self.dw = bf(M, N), bf(M, K), bf(N, K)
        self.sc = torch.zeros(16, dtype=torch.float32, device=dev)
        self.saved = tw.make_saved(self.xq, self.xqT, self.wq, self.wqT, self.sc)
        self.S = torch.zeros(2, dtype=torch.float64, device=dev)
        self.ws = torch.empty(max(tw.tweo_workspace_bytes(op, M, N, K) for op in
                                  (tw.TWEO_OP_FP8_LINEAR_FWD_BF16, tw.TWEO_OP_FP8_LINEAR_BWD_BF16)),
                              dtype=torch.uint8, device=dev)
        self.flops = 6.0 * M * N * K
        # delayed-scaling states of the three scaled tensors (x, w, dy)
        self.st = [torch.zeros(tw.DELAYED_STATE_WORDS, dtype=torch.float32, device=dev) for _ in range(3)]


def run_step(tw, layers, ev=None):
    """The whole path through the two bf16 entry points: amax and casts of X and W, forward GEMM
    with the penalty epilogue and its finishing sum; amax and cast of dY, dgrad and wgrad GEMMs.
    `ev`: the three GEMM kernels of every layer record their own start and end events."""
    # the order of a training step: every forward, then the backwards from the last layer down
    for L in layers:
        if ev is not None:
            ev.arm(1, 2.0 * L.M * L.N * L.K)
        tw.tweo_fp8_linear_fwd_bf16(L.x, L.w, L.y, L.saved, pen=PEN, penalty_sum=L.S, workspace=L.ws)
    for L in reversed(layers):
        if ev is not None:
            ev.arm(2, 2.0 * L.M * L.N * L.K)
        tw.tweo_fp8_linear_bwd_bf16(L.dy, L.saved, L.K, L.dyq, L.dyqT, L.dx, L.dw, L.ws)


def run_step_delayed(tw, layers, bootstrap=False, hybrid=False):
    """The same step under the paper's own recipe (Sec. 4.3): delayed scaling, every tensor cast in
    one pass with the scale its amax history fixed beforehand, no separate amax pass, through
    tweo_fp8_linear_fwd_bf16_delayed / tweo_fp8_linear_bwd_bf16_delayed.  hybrid: the gradient is
    cast to E5M2 as in the paper's HYBRID format."""
    for L in layers:
        sx, sw, sdy = L.st
        tw.tweo_fp8_linear_fwd_bf16_delayed(L.x, L.w, L.y, L.saved, sx, sw, bootstrap=bootstrap, pen=PEN,
                                            penalty_sum=L.S, workspace=L.ws)
    for L in reversed(layers):
        sx, sw, sdy = L.st
        tw.tweo_fp8_linear_bwd_bf16_delayed(L.dy, L.saved, sdy, L.K, L.dyq, L.dyqT, L.dx, L.dw, L.ws,
                                            bootstrap=bootstrap, dy_e5m2=hybrid)


class GemmEvents:
    """HIP events that the GEMM kernels of the timed steps record at their own start and end
    (tweo_profile_gemm_launches: hipExtLaunchKernelGGL on the launch stream), so that a pair
    times one kernel launch, like a profiler's kernel trace does, without draining the stream."""

    def __init__(self, torch, tw):
        self.torch, self.tw, self.pairs, self.flops = torch, tw, [], []

    def _event(self):
        e = self.torch.cuda.Event(enable_timing=True)
        e.record()  # creates the handle
        return e

    def arm(self, launches, flops_each):
        evs = []
        for _ in range(launches):
            s, e = self._event(), self._event()
            self.pairs.append((s, e))
            self.flops.append(flops_each)
            evs += [s.cuda_event, e.cuda_event]
        self.tw.tweo_profile_gemm_launches(evs)

    def durations_ms(self):
        return [s.elapsed_time(e) for s, e in self.pairs]


def time_elementwise(tw, torch, L, peers, iters=20):
    """GB/s of the amax and quantize passes on this layer's largest activation (algorithmic bytes).
    warm: the same tensor again and again (184 MB: it stays in the 256 MB memory-side cache, so
    this is NOT an HBM figure).  cold: the passes rotate over `peers` + this tensor, at least
    four distinct tensors of the same shape whose total is several times the cache, with
    output buffers rotating too, so that every byte comes from / goes to HBM."""
    out = {}
    n = L.M * L.K
    xs = [L.x] + peers
    assert len(xs) >= 3 and all(t.numel() == n for t in xs)
    qs = [torch.empty((L.M, L.K), dtype=torch.uint8, device=L.x.device) for _ in xs]
    qTs = [torch.empty((L.K, L.M), dtype=torch.uint8, device=L.x.device) for _ in xs]
    xs = [t.view(L.M, L.K) for t in xs]
    am = torch.zeros(4 * len(xs), dtype=torch.float32, device=L.x.device)
    for i, t in enumerate(xs):
        tw.tweo_amax(t, am[4 * i:4 * i + 1])
    sc = torch.zeros(8, dtype=torch.float32, device=L.x.device)
    slots = torch.empty(4096, dtype=torch.uint8, device=L.x.device)
    # amax + cast + transposed copy in one call: 4 algorithmic bytes per element (one read, two
    # writes); two launches move 6 (the one-launch form re-reads what it cannot keep on chip)
    passes = (
        ("amax", lambda i: tw.tweo_amax(xs[i], am[4 * i:4 * i + 1]), 2.0),
        ("quantize_e4m3_T", lambda i: tw.tweo_quantize_e4m3(xs[i], am[4 * i:4 * i + 1], qs[i], qTs[i]), 4.0),
        ("quantize_e4m3", lambda i: tw.tweo_quantize_e4m3(xs[i], am[4 * i:4 * i + 1], qs[i], None), 3.0),
        ("amax_quantize_T_one_call", lambda i: tw.tweo_amax_quantize_f8(xs[i], sc[0:1], qs[i], qTs[i], sc[4:5], sc[5:6], slots), 4.0),
        # static INT8 quantisation (Eq. 4 with a precomputed step): 2 read + 1 written
        ("quantize_i8_static", lambda i: tw.tweo_quantize_i8(xs[i], 127.0 / 20.0, qs[i].view(torch.int8)), 3.0))
    for name, fn, bytes_per_elt in passes:
        res = {"MB": round(n * bytes_per_elt / 1e6, 1)}
        for mode, pick in (("warm", lambda k: 0), ("cold", lambda k: k % len(xs))):
            for k in range(len(xs)):
                fn(pick(k))
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            for k in range(iters):
                fn(pick(k))
            e.record()
            torch.cuda.synchronize()
            ms = s.elapsed_time(e) / iters
            res[mode] = {"GB/s": round(n * bytes_per_elt / ms / 1e6, 1), "us": round(ms * 1e3, 2),
                         "frac_of_hbm_peak": round(n * bytes_per_elt / ms / 1e6 / HBM_PEAK_GBS, 3)}
        out[name] = res
    # the reduction kernel alone (its own start-to-end events, no clearing launch in front): a pure
    # read of the tensor, i.e. what one kernel can stream from HBM on this machine
    ev = GemmEvents(torch, tw)
    d = []
    for lo in range(0, 16, 8):
        ev = GemmEvents(torch, tw)
        ev.arm(8, 0.0)
        for k in range(8):
            tw.tweo_amax(xs[(lo + k) % len(xs)], am[0:1])
        torch.cuda.synchronize()
        d += ev.durations_ms()
    us = sorted(d)[len(d) // 2] * 1e3
    out["amax"]["cold_kernel_only"] = {"us": round(us, 2), "GB/s": round(2.0 * n / us / 1e3, 1),
                                       "frac_of_hbm_peak": round(2.0 * n / us / 1e3 / HBM_PEAK_GBS, 3)}
    out["note"] = "cold = rotation over %d distinct %.0f MB tensors (HBM); warm = one tensor (memory-side cache)" % (
        len(xs), n * 2 / 1e6)
    return out


def time_layernorm(tw, torch, dev, rows=16384, cols=2048, copies=6, iters=24):
    """LayerNorm -> E4M3 cast (+ transposed copy) of a residual stream of the workload's shape
    (Sec. 4.3: LayerNorm runs under FP8 too), cold: the calls rotate over `copies` distinct
    tensors (6 x 67 MB against 256 MB of memory-side cache).  Algorithmic bytes: 2 read + 1 + 1
    written per element; beside it the plain amax + cast of the same tensors (the same bytes)."""
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    xs = [(torch.randn((rows, cols), device=dev, generator=g) * 3).to(torch.bfloat16) for _ in range(copies)]
    gamma = (1 + 0.1 * torch.randn((cols,), device=dev, generator=g)).to(torch.bfloat16)
    beta = (0.1 * torch.randn((cols,), device=dev, generator=g)).to(torch.bfloat16)
    qs = [torch.empty((rows, cols), dtype=torch.uint8, device=dev) for _ in range(copies)]
    qTs = [torch.empty((cols, rows), dtype=torch.uint8, device=dev) for _ in range(copies)]
    ws = torch.empty(tw.tweo_workspace_bytes(tw.TWEO_OP_LAYERNORM_QUANTIZE, rows, 1, 1), dtype=torch.uint8, device=dev)
    st = torch.zeros(tw.DELAYED_STATE_WORDS, dtype=torch.float32, device=dev)
    am = torch.zeros(4, dtype=torch.float32, device=dev)
    tw.tweo_delayed_state_init(st)
    tw.tweo_layernorm_quantize_e4m3_delayed(xs[0], gamma, st, qs[0], ws, bootstrap=True, beta_bf16=beta, qT=qTs[0])

    def plain(i):
        tw.tweo_amax(xs[i], am[0:1])
        tw.tweo_quantize_e4m3(xs[i], am[0:1], qs[i], qTs[i])

    forms = (("layernorm_cast_current_scaling", lambda i: tw.tweo_layernorm_quantize_e4m3(
                 xs[i], gamma, qs[i], ws, beta_bf16=beta, qT=qTs[i])),
             ("layernorm_cast_delayed_scaling", lambda i: tw.tweo_layernorm_quantize_e4m3_delayed(
                 xs[i], gamma, st, qs[i], ws, beta_bf16=beta, qT=qTs[i])),
             ("amax_plus_cast_no_layernorm", plain))
    out = {"tensor": "%dx%d bf16, %d copies" % (rows, cols, copies)}
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, fn in forms:
        for k in range(copies):
            fn(k)
        s.record()
        for k in range(iters):
            fn(k % copies)
        e.record()
        torch.cuda.synchronize()
        us = s.elapsed_time(e) / iters * 1e3
        out[name] = {"us": round(us, 2), "GB/s": round(4.0 * rows * cols / us / 1e3, 1),
                     "frac_of_hbm_peak": round(4.0 * rows * cols / us / 1e3 / HBM_PEAK_GBS, 3)}
    return out


def vendor_library_context(torch, layers, reps=6):
    """Context, not a product path: the FP8 GEMM of the vendor's library (hipBLASLt behind
    torch._scaled_mm) on the same 15 GEMMs, fed with the codes the step above left in the layers'
    buffers, each launch timed by its own pair of events.  Shows what fraction of the datasheet
    peak a tuned library kernel reaches on this machine under the same operand statistics."""
    try:
        f8 = torch.float8_e4m3fn
        one = torch.ones((), dtype=torch.float32, device=layers[0].xq.device)
        calls = []
        for L in layers:
            fl = 2.0 * L.M * L.N * L.K
            calls += [("%s fwd" % L.name, L.xq, L.wq, fl), ("%s dgrad" % L.name, L.dyq, L.wqT, fl),
                      ("%s wgrad" % L.name, L.dyqT, L.xqT, fl)]
        mm = lambda a, b: torch._scaled_mm(a.view(f8), b.view(f8).t(), scale_a=one, scale_b=one,
                                           out_dtype=torch.bfloat16)
        for _ in range(2):
            for _, a, b, _ in calls:
                mm(a, b)
        torch.cuda.synchronize()
        evs = []
        for _ in range(reps):
            for _, a, b, _ in calls:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                mm(a, b)
                e1.record()
                evs.append((e0, e1))
        torch.cuda.synchronize()
        us = [1e3 * e0.elapsed_time(e1) for e0, e1 in evs]
        per = {}
        for i, (name, _, _, fl) in enumerate(calls):
            d = sorted(us[i::len(calls)])[reps // 2]
            per[name] = {"us": round(d, 1), "TFLOP/s": round(fl / d / 1e6, 1)}
        tot_us = sum(v["us"] for v in per.values())
        tot_fl = sum(c[3] for c in calls)
        return {"what": "torch._scaled_mm (vendor FP8 GEMM library) on the same 15 GEMMs and operand codes; "
                        "medians of %d event-timed calls each, events around the call" % reps,
                "TFLOP/s": round(tot_fl / tot_us / 1e6, 1),
                "frac_of_fp8_peak": round(tot_fl / tot_us / 1e6 / FP8_PEAK_TFLOPS, 4), "per_gemm": per}
    except Exception as e:  # a context figure: its absence must not fail the bench
        return {"error": "%s: %s" % (type(e).__name__, str(e)[:200])}


def time_penalty_cost(tw, torch, L, reps=24):
    """What the fused penalty (Sec. 3.3) costs on one layer's forward GEMM, operands already
    quantised, with and without, alternating, medians.  Two clocks: the GEMM kernel's own
    start-to-end events (the epilogue arithmetic only), and stream events around batches of
    calls (everything the penalty adds: the epilogue and the finishing launch)."""
    inv = lambda i: L.sc[i:i + 1]

    def call(with_pen):
        if with_pen:
            tw.tweo_fp8_linear_fwd(L.xq, inv(2), L.wq, inv(5), L.y, pen=PEN, penalty_sum=L.S, workspace=L.ws)
        else:
            tw.tweo_fp8_linear_fwd(L.xq, inv(2), L.wq, inv(5), L.y, workspace=L.ws)

    t = {True: [], False: []}
    tc = {True: [], False: []}
    for _ in range(reps // 8):
        for with_pen in (True, False, False, True):
            ev = GemmEvents(torch, tw)
            ev.arm(2, 0.0)
            for _ in range(2):
                call(with_pen)
            torch.cuda.synchronize()
            t[with_pen] += ev.durations_ms()
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            for _ in range(8):
                call(with_pen)
            e.record()
            torch.cuda.synchronize()
            tc[with_pen].append(s.elapsed_time(e) / 8)
    med = lambda v: sorted(v)[len(v) // 2] * 1e3
    return {"layer": "%s %dx%dx%d" % (L.name, L.M, L.K, L.N),
            "gemm_kernel_with_penalty_us": round(med(t[True]), 2), "gemm_kernel_without_us": round(med(t[False]), 2),
            "call_with_penalty_us": round(med(tc[True]), 2), "call_without_us": round(med(tc[False]), 2),
            "note": "call_* = back-to-back calls timed by stream events, finishing launch of the penalty included"}


def time_w8a8(tw, torch, synth, dev, iters=20, copies=8):
    """W8A8 INT8 inference GEMMs at the 7B shapes (Sec. 4.4): qkv 4096->12288, gate and up
    4096->11008, down 11008->4096, for M in {1, 16, 64, 4096}, on the workload's own statistics
    (N(0,1) activations clipped at 20, N(0,0.02) weights, per-tensor static steps amax/127).
    M <= 64 is bound by streaming the weights: a decode step reads each layer's weights once, so
    the figure that counts is COLD - the call rotates over `copies` distinct weight matrices
    (row-rotated copies of the quantised weights, 360-400 MB in total against 256 MB of
    memory-side cache); the warm figure (one 45-50 MB matrix, cache resident) is printed beside it."""
    res = {}
    up = lambda b: torch.from_numpy(b.view("int16")).to(dev).view(torch.bfloat16)

    def quant(t):
        amax = float(t.float().abs().max())
        q = torch.empty(t.shape, dtype=torch.int8, device=dev)
        tw.tweo_quantize_i8(t, 127.0 / amax, q)
        return q, amax / 127.0

    def kernel_us(fns):
        # the kernels' own start-to-end times (events recorded by the launches themselves)
        d = []
        for lo in range(0, len(fns), 8):  # as many as the hook holds at a time
            ev = GemmEvents(torch, tw)
            ev.arm(len(fns[lo:lo + 8]), 0.0)
            for fn in fns[lo:lo + 8]:
                fn()
            torch.cuda.synchronize()
            d += ev.durations_ms()
        d = sorted(d)
        return d[len(d) // 2] * 1e3

    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def stream_us(fns, n_warm):
        for k in range(n_warm):
            fns[k % len(fns)]()
        s.record()
        for k in range(iters):
            fns[k % len(fns)]()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / iters * 1e3

    for gi, g in enumerate(synth.CONFIGS[4]["gemms"]):
        K, N = g.K, g.N
        shape = {}
        wqs = None
        for M in (1, 16, 64, 128, 512, 4096):  # 128 and 512: between the sizes the workload names
            x, w = synth.w8a8_inputs(gi, M, with_w=wqs is None)
            if wqs is None:
                wq, step_w = quant(up(w))
                wqs = [wq] + [torch.roll(wq, 16 * 37 * (c + 1), 0) for c in range(copies - 1)]
            if "plain_read_of_the_weights_cold" not in shape:
                # what ONE kernel needs to read these bytes cold, doing nothing else: the amax
                # reduction kernel (its own events) over the same rotating copies
                am = torch.zeros(4, dtype=torch.float32, device=dev)
                reads = [(lambda c: (lambda: tw.tweo_amax(wqs[c].view(torch.bfloat16), am[0:1])))(c) for c in range(copies)]
                us_r = kernel_us(reads + reads)
                shape["plain_read_of_the_weights_cold"] = {"us": round(us_r, 2), "GB/s": round(N * K / us_r / 1e3, 1)}
            xq, step_x = quant(up(x))
            ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(copies if M <= 128 else 1)]
            ws = torch.empty(tw.tweo_workspace_bytes(tw.TWEO_OP_W8A8_LINEAR, M, N, K), dtype=torch.uint8, device=dev)
            bytes_ = M * K + N * K + 2 * M * N
            call = lambda c: (lambda: tw.tweo_w8a8_linear(xq, wqs[c], step_x * step_w, ys[c % len(ys)], ws))
            r = {}
            if M <= 128:  # the weight-streaming kernel
                warm, cold = [call(0)] * 8, [call(c) for c in range(copies)]
                stream_us(cold, copies)
                r["cold_kernel_us"] = round(kernel_us(cold + cold), 2)
                r["cold_GB/s"] = round(bytes_ / r["cold_kernel_us"] / 1e3, 1)
                r["cold_frac_of_hbm_peak"] = round(r["cold_GB/s"] / HBM_PEAK_GBS, 3)
                r["cold_call_us"] = round(stream_us(cold, copies), 2)
                stream_us(warm, 3)
                r["warm_kernel_us"] = round(kernel_us(warm), 2)
                r["warm_GB/s"] = round(bytes_ / r["warm_kernel_us"] / 1e3, 1)
            else:
                # the compute-bound shape is timed at the clock the chip settles at under load: it
                # takes some 20 ms of work to get there from the idle state the small shapes leave
                us = stream_us([call(c) for c in range(copies)] if M < 4096 else [call(0)], 100)  # weights cold below 4096
                r["us"] = round(us, 2)
                r["TOP/s"] = round(2.0 * M * N * K / us / 1e6, 2)
                r["frac_of_int8_peak"] = round(2.0 * M * N * K / us / 1e6 / INT8_PEAK_TOPS, 3)
                try:
                    # context, not a path of this library: the vendor library's INT8 GEMM on the same
                    # codes (int32 output, no dequantisation), timed the same way
                    wt = wqs[0].t()
                    us_v = stream_us([lambda: torch._int_mm(xq, wt)], 100)
                    r["vendor_int_mm_context"] = {"us": round(us_v, 2), "TOP/s": round(2.0 * M * N * K / us_v / 1e6, 2)}
                except Exception as ex:
                    r["vendor_int_mm_context"] = {"error": "%s: %s" % (type(ex).__name__, str(ex)[:120])}
            shape["M=%d" % M] = r
            if gi == 0 and M in (1, 16, 64, 4096):
                # the finer granularities of Sec. 4.4 on the same codes: per-token steps found on the
                # fly (quantise kernel timed with the GEMM), per-channel weight steps
                xb = up(x)
                xq2 = torch.empty((M, K), dtype=torch.int8, device=dev)
                sx = torch.empty((M,), dtype=torch.float32, device=dev)
                sw = torch.full((N,), step_w, dtype=torch.float32, device=dev)
                n_warm = 3 if M <= 64 else 50
                us_q = stream_us([lambda: tw.tweo_quantize_i8_rows(xb, 1e-6, xq2, sx)], n_warm)
                gemm = [(lambda c: (lambda: tw.tweo_w8a8_linear_scaled(xq2, wqs[c], sx, sw, ys[c % len(ys)])))(c)
                        for c in range(copies if M <= 64 else 1)]
                us_g = stream_us(gemm, n_warm)
                fine = {"quantize_rows_us": round(us_q, 2), "gemm_call_us_cold": round(us_g, 2),
                        "gemm_kernel_us_cold": round(kernel_us(gemm + gemm), 2)}
                if M <= 64:
                    # the decode step (per-token quantise + GEMM) as one HIP graph: what the pair costs
                    # once the host's per-call time is out of the way (cold weights: the graph
                    # holds one pair per weight copy)
                    pairs = lambda: [(tw.tweo_quantize_i8_rows(xb, 1e-6, xq2, sx), f()) for f in gemm]
                    side = torch.cuda.Stream()
                    side.wait_stream(torch.cuda.current_stream())
                    with torch.cuda.stream(side):
                        pairs()
                    torch.cuda.current_stream().wait_stream(side)
                    torch.cuda.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=side):
                        pairs()
                    fine["quantize_plus_gemm_in_graph_us_cold"] = round(stream_us([graph.replay], 2) / len(gemm), 2)
                r["W(C)A(K)"] = fine
        res["%s %d->%d" % (g.name, K, N)] = shape
        del wqs
        torch.cuda.empty_cache()
    return res


def cpu_baseline(synth, cfg, host=None, target_s=5.0):
    """The CPU oracle, as it stands, on a bounded row sample of the first GEMM of the workload."""
    import numpy as np
    import oracle
    g = synth.CONFIGS[cfg]["gemms"][0]
    M, K, N = g.M, g.K, g.N
    x, w, dy = host if host is not None else synth.fp8_linear_inputs(cfg, 0)
    rows_q = min(M, 8192)

    def quant(t):
        s, si = oracle.scale_from_amax(oracle.amax_bf16(t))
        q, _ = oracle.quantize_e4m3(t, s, transpose=False)
        return q, si

    t0 = time.perf_counter()
    xq, sxi = quant(x[:rows_q])
    wq, swi = quant(w)
    dyq, sdyi = quant(dy[:rows_q])
    t_cast = time.perf_counter() - t0
    # calibrate on a few rows, then size each GEMM leg for about target_s seconds
    probe = np.arange(0, min(rows_q, 16))
    t0 = time.perf_counter()
    oracle.fp8_linear_fwd(xq, wq, sxi, swi, rows=probe, want_abs=False)
    per_row = (time.perf_counter() - t0) / len(probe)
    r = int(max(16, min(rows_q, target_s / max(per_row, 1e-9))))
    rows = np.arange(r)
    t0 = time.perf_counter()
    oracle.fp8_linear_fwd(xq, wq, sxi, swi, rows=rows, want_abs=False)
    oracle.fp8_linear_dgrad(dyq, wq, sdyi, swi, rows=rows, want_abs=False)
    rn = min(N, max(8, r * N // rows_q))  # same flop count as one of the other two legs
    oracle.fp8_linear_wgrad(dyq, xq, sdyi, sxi, rows=np.arange(rn), want_abs=False)
    t_gemm = time.perf_counter() - t0
    flops = 2.0 * r * N * K * 2 + 2.0 * rn * rows_q * K
    return {"value": round(flops / t_gemm / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "%s: fp64 oracle fwd+dgrad on %d rows of M, wgrad on %d rows of N over %d "
                      "tokens (%.1f s); casts of those rows %.2f s not included"
                      % (g.name, r, rn, rows_q, t_gemm, t_cast)}


def profiled_traffic(workload):
    """HBM-side bytes per GEMM launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs of this command, scaled by a plain copy); only known for the default workload."""
    if workload != "llama" or not os.path.exists(PROFILE_TRAFFIC):
        return None
    for line in open(PROFILE_TRAFFIC):
        if line.startswith("gemm_traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


EVENT_EVERY = 10  # an instrumented step is ~6 % slower (a gap opens in front of each of its 15 GEMM kernels)


def time_workload(tw, torch, synth, cfg, dev, steps, warmup):
    """ms per step, end-to-end TFLOP/s and GEMM-kernel TFLOP/s of another workload (same step)."""
    layers = [Layer(tw, torch, synth, cfg, gi, dev) for gi in range(len(synth.CONFIGS[cfg]["gemms"]))]
    for L in layers:
        L.host = None
    flops = sum(L.flops for L in layers)
    for _ in range(warmup):
        run_step(tw, layers)
    torch.cuda.synchronize()
    ev = GemmEvents(torch, tw)
    t0 = time.perf_counter()
    for i in range(steps):
        run_step(tw, layers, ev if i % EVENT_EVERY == 0 else None)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    # a few more steps timed by stream events: at sub-millisecond steps the host's launch time shows in the wall clock
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(steps):
        run_step(tw, layers)
    e.record()
    torch.cuda.synchronize()
    gemm_ms = sum(ev.durations_ms())
    res = {"workload": synth.CONFIGS[cfg]["name"], "ms_per_step": round(ms, 4),
           "ms_per_step_stream_events": round(s.elapsed_time(e) / steps, 4),
           "TFLOP/s": round(flops / ms / 1e9, 2),
           "gemm_TFLOP/s": round(sum(ev.flops) / gemm_ms / 1e9, 2),
           "gemm_frac_of_fp8_peak": round(sum(ev.flops) / gemm_ms / 1e9 / FP8_PEAK_TFLOPS, 4),
           "gemm_launches": len(ev.pairs)}
    if ms < 1.0:
        # launch-bound steps: the same step captured once into a HIP graph and replayed (under
        # capture the entry points record the two-launch form of every cast)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run_step(tw, layers)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run_step(tw, layers)
        for _ in range(warmup):
            graph.replay()
        s.record()
        for _ in range(steps):
            graph.replay()
        e.record()
        torch.cuda.synchronize()
        res["ms_per_step_replayed_hip_graph"] = round(s.elapsed_time(e) / steps, 4)
        res["TFLOP/s_replayed_hip_graph"] = round(flops / (s.elapsed_time(e) / steps) / 1e9, 2)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--tile", type=int, default=0, help="force a GEMM kernel variant (0 = heuristic)")
    ap.add_argument("--stream-k", action="store_true",
                    help="switch the K-split of partial last rounds of tiles on")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of 256 MiB (for scaling rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (the path has no multi-GPU part); "
            "--gpus %d is not supported" % a.gpus)
        sys.exit(2)

    import torch
    import paper_2511_23225_amd as tw
    from paper_2511_23225_amd import synth
    if not os.path.exists(tw.LIB_PATH):
        from paper_2511_23225_amd import build as b
        b.build_library()
    tw.load()
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    dev = "cuda:0"
    if a.copy_calibration:
        n = 256 << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(max(1, a.steps)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_each_way": n, "copies": max(1, a.steps)}), flush=True)
        return
    cfg = WORKLOADS[a.workload]
    tw.tweo_set_stream_k(a.stream_k)  # before the workspaces are sized
    t0 = time.perf_counter()
    layers = [Layer(tw, torch, synth, cfg, gi, dev) for gi in range(len(synth.CONFIGS[cfg]["gemms"]))]
    log("inputs generated and uploaded in %.1f s" % (time.perf_counter() - t0))
    tw.tweo_set_gemm_tile(a.tile)
    step_flops = sum(L.flops for L in layers)
    host0 = layers[0].host
    for L in layers:
        L.host = None

    for _ in range(a.warmup):
        run_step(tw, layers)
    torch.cuda.synchronize()
    # The GEMM kernels of every EVENT_EVERY-th timed step record their own start/end events.
    ev = GemmEvents(torch, tw)
    t0 = time.perf_counter()
    for i in range(a.steps):
        run_step(tw, layers, ev if i % EVENT_EVERY == 0 else None)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / a.steps
    dur = ev.durations_ms()
    gemm_ms = sum(dur)
    # per-kernel detail on stderr: three launches per layer per timed step (fwd, dgrad, wgrad)
    per_step = 3 * len(layers)
    for li, L in enumerate(layers):
        fl = 2.0 * L.M * L.N * L.K
        parts = []
        nl = len(layers)
        # order of the launches inside a step: the forwards of layers 0..n-1, then (dgrad, wgrad) of
        # layers n-1..0
        where = {"fwd": li, "dgrad": nl + 2 * (nl - 1 - li), "wgrad": nl + 2 * (nl - 1 - li) + 1}
        for name in ("fwd", "dgrad", "wgrad"):
            d = [dur[j] for j in range(len(dur)) if j % per_step == where[name]]
            parts.append("%s %7.1f us %5.0f TFLOP/s" % (name, 1e3 * sum(d) / len(d), fl / (sum(d) / len(d)) / 1e9))
        log("  %-5s %s" % (L.name, "   ".join(parts)))
    n_gemm_launches = len(dur)
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    gemm_tflops = sum(ev.flops) / (gemm_ms * 1e-3) / 1e12

    out = {
        "metric": "FP8 linear fwd+bwd TFLOP/s (+penalty), end to end from bf16 operands",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3 (fp32 accumulate)",
        "data": "synthetic",
        "config": {"workload": synth.CONFIGS[cfg]["name"],
                   "gemms": ["%s %dx%dx%d" % (L.name, L.M, L.K, L.N) for L in layers],
                   "flop_per_step": step_flops, "penalty": "tau=3 p=4 eps=1e-6, fused",
                   "tile": a.tile},
        "roofline": {"bound": "mfma", "kernel": "gemm_nt_defer_kernel (fp8 fwd, dgrad, wgrad; tile-starved ones: other variants or a K split)",
                     "achieved": round(gemm_tflops, 2), "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / FP8_PEAK_TFLOPS, 4),
                     "traffic": profiled_traffic(a.workload) if a.tile == 0 else None,
                     "traffic_source": "committed rocprofv3 --pmc summary of this command "
                                       "(profiles/fp8_gemm_llama_block_pmc_traffic.txt), not measured by this run",
                     "algorithmic_bytes_per_launch": round(
                         sum((L.M * L.K + L.N * L.K + 2 * L.M * L.N) + (L.M * L.N + L.N * L.K + 2 * L.M * L.K)
                             + (L.M * L.N + L.M * L.K + 2 * L.N * L.K) for L in layers) / (3.0 * len(layers))),
                     "flop_per_launch": round(step_flops / (3.0 * len(layers))),
                     "avg_launch_us": round(gemm_ms * 1e3 / n_gemm_launches, 2),
                     "launches": n_gemm_launches},
        "pct_of_fp8_peak_end_to_end": round(100.0 * value / FP8_PEAK_TFLOPS, 2),
        "paper_context": "+36% training throughput FP8 over BF16 (hardware unstated)",
    }
    if not a.no_extras:
        # the paper's own scaling mode, same step otherwise (reported beside, never as `value`)
        for L in layers:
            for st in L.st:
                tw.tweo_delayed_state_init(st)
        run_step_delayed(tw, layers, bootstrap=True)
        for _ in range(2):
            run_step_delayed(tw, layers)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            run_step_delayed(tw, layers)
        torch.cuda.synchronize()
        ms_d = (time.perf_counter() - t0) * 1e3 / a.steps
        out["delayed_scaling_history16"] = {"ms_per_step": round(ms_d, 4),
                                            "TFLOP/s": round(step_flops / (ms_d * 1e-3) / 1e12, 2)}
        # the paper's recipe in full: delayed scaling and E5M2 gradients (fresh gradient states)
        for L in layers:
            tw.tweo_delayed_state_init(L.st[2])
        run_step_delayed(tw, layers, bootstrap=True, hybrid=True)
        for _ in range(2):
            run_step_delayed(tw, layers, hybrid=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            run_step_delayed(tw, layers, hybrid=True)
        torch.cuda.synchronize()
        ms_h = (time.perf_counter() - t0) * 1e3 / a.steps
        out["delayed_scaling_hybrid_e5m2_gradients"] = {"ms_per_step": round(ms_h, 4),
                                                        "TFLOP/s": round(step_flops / (ms_h * 1e-3) / 1e12, 2)}
        if a.workload == "llama":
            out["vendor_library_context"] = vendor_library_context(torch, layers)
        big = max(layers, key=lambda L: L.M * L.K)
        peers = [L.y for L in layers if L is not big and L.y.numel() == big.x.numel()]
        while len(peers) < 3:
            peers.append(torch.roll(big.x.view(-1), 12345 * (len(peers) + 1)).view_as(big.x))
        out["elementwise"] = time_elementwise(tw, torch, big, peers)
        out["elementwise"]["peak_GB/s"] = HBM_PEAK_GBS
        del peers
        out["penalty_cost"] = time_penalty_cost(tw, torch, layers[0])
        out["layernorm"] = time_layernorm(tw, torch, dev)
        del layers, big
        torch.cuda.empty_cache()
        out["w8a8_7b"] = time_w8a8(tw, torch, synth, dev)
        out["other_workloads"] = {}
        for name in ("gpt2", "vit", "single"):
            if name != a.workload:
                out["other_workloads"][name] = time_workload(tw, torch, synth, WORKLOADS[name], dev, a.steps, a.warmup)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth, cfg, host0)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
