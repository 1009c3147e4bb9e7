"""The entry points allocate nothing, clear nothing with memset nodes and never synchronise, so a
caller can capture them in a HIP graph.  Each graph is replayed several times with new data in
the same buffers, with eager work and synchronisations in between, and every replay must give
the bits the eager calls give for the same data (the kernels are run-to-run deterministic)."""
import numpy as np
import pytest
import torch

import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, PEN, to_dev_bf16

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def test_fp8_linear_step_in_a_graph():
    M, K, N = 256, 512, 512
    say("graph: fp8 linear fwd+bwd M=%d K=%d N=%d" % (M, K, N))
    datasets = [synth.fp8_linear_inputs(0, 0)]
    x0, w0, dy0 = datasets[0]
    rng = np.random.default_rng(11)
    for _ in range(2):  # other data of the same shape: permuted rows, so amax and every byte move
        datasets.append((x0[rng.permutation(M)], w0[rng.permutation(N)], dy0[rng.permutation(M)]))
    u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=DEV)
    bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=DEV)
    x, w, dy = bf(M, K), bf(N, K), bf(M, N)
    xq, xqT, wq, wqT, dyq, dyqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N), u8(M, N), u8(N, M)
    sc = torch.zeros(16, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    y, dx, dw = bf(M, N), bf(M, K), bf(N, K)
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    ws = torch.empty(max(tw.tweo_workspace_bytes(op, M, N, K) for op in
                         (tw.TWEO_OP_FP8_LINEAR_FWD_BF16, tw.TWEO_OP_FP8_LINEAR_BWD_BF16)),
                     dtype=torch.uint8, device=DEV)

    def step():
        tw.tweo_fp8_linear_fwd_bf16(x, w, y, saved, pen=PEN, penalty_sum=S, workspace=ws)
        tw.tweo_fp8_linear_bwd_bf16(dy, saved, K, dyq, dyqT, dx, dw, ws)

    def load(d):
        x.copy_(to_dev_bf16(d[0])); w.copy_(to_dev_bf16(d[1])); dy.copy_(to_dev_bf16(d[2]))

    def outputs():
        torch.cuda.synchronize()
        return [t.clone() for t in (y.view(torch.int16), dx.view(torch.int16), dw.view(torch.int16), S, sc, dyq)]

    eager = []
    for d in datasets:
        load(d)
        step()
        eager.append(outputs())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(2):
        for i, d in enumerate(datasets):
            load(d)
            for t in (y, dx, dw):
                t.fill_(float("nan"))  # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            got = outputs()
            for name, a, b in zip(("y", "dx", "dw", "S", "scalars", "dyq"), got, eager[i]):
                assert torch.equal(a, b), "replay %d of dataset %d: %s differs from the eager result in %d of %d" % (
                    rep, i, name, int((a != b).sum()), a.numel())


def test_w8a8_decode_step_in_a_graph():
    M, K, N = 16, 1024, 8192
    say("graph: per-token quantise + W8A8 linear M=%d K=%d N=%d" % (M, K, N))
    datasets = [synth.w8a8_inputs(0, M, K=K, N=N)[0]]
    rng = np.random.default_rng(5)
    datasets += [datasets[0][rng.permutation(M)][:, rng.permutation(K)] for _ in range(2)]
    _, wb = synth.w8a8_inputs(0, M, K=K, N=N)
    wq = torch.empty((N, K), dtype=torch.int8, device=DEV)
    sw = torch.empty((N,), dtype=torch.float32, device=DEV)
    tw.tweo_quantize_i8_rows(to_dev_bf16(wb), 1e-6, wq, sw)  # weights per channel, offline
    x = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=DEV)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)

    def step():
        tw.tweo_quantize_i8_rows(x, 1e-6, xq, sx)
        tw.tweo_w8a8_linear_scaled(xq, wq, sx, sw, y)

    eager = []
    for d in datasets:
        x.copy_(to_dev_bf16(d))
        step()
        torch.cuda.synchronize()
        eager.append(y.view(torch.int16).clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(2):
        for i, d in enumerate(datasets):
            x.copy_(to_dev_bf16(d))
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), eager[i]), "replay %d of dataset %d" % (rep, i)
