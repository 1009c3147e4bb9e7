"""GPU parity of the one-launch amax + cast of the bf16 entry points (Sec. 4.3, current scaling:
one scale per tensor from the tensor's own amax): codes, transposed codes, amax and scales against
the oracle bit for bit, and against the two-launch form of the same entry points, for one and two
tensors per launch, one to three rounds of blocks per workgroup, edges that end inside a 256x256
tile, both gradient formats, a NaN and an all-zero tensor."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, PEN, to_dev_bf16, bf16_bits, workspace

pytestmark = pytest.mark.gpu


def run_step(x, w, dy, M, K, N, fused, dy_e5m2):
    u8 = lambda *s: torch.full(s, 0x55, dtype=torch.uint8, device=DEV)
    xq, xqT, wq, wqT, dyq, dyqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N), u8(M, N), u8(N, M)
    sc = torch.full((16,), -3.0, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    dx = torch.full((M, K), float("nan"), dtype=torch.bfloat16, device=DEV)
    dw = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device=DEV)
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD_BF16, M, N, K)
    wsb = workspace(tw.TWEO_OP_FP8_LINEAR_BWD_BF16, M, N, K)
    ws.fill_(0xA5)   # whatever an earlier call left behind must not matter
    wsb.fill_(0xA5)
    tw.tweo_set_fused_cast(fused)
    try:
        tw.tweo_fp8_linear_fwd_bf16(x, w, y, saved, pen=PEN, penalty_sum=S, workspace=ws)
        bwd = tw.tweo_fp8_linear_bwd_bf16_hybrid if dy_e5m2 else tw.tweo_fp8_linear_bwd_bf16
        bwd(dy, saved, K, dyq, dyqT, dx, dw, wsb)
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_fused_cast(True)
    codes = [t.cpu().numpy() for t in (xq, xqT, wq, wqT, dyq, dyqT)]
    return codes, sc.cpu().numpy()[:9].copy(), [bf16_bits(t) for t in (y, dx, dw)], float(S.cpu()[0])


# M, K, N (the one-launch form takes tensors from 2^24 elements): (a) one round of blocks per
# workgroup, every edge inside a tile; (b) the activation fills two rounds of 256 workgroups x 8
# waves, the gradient three; (c) two tensors of unequal size, the small one first (the gradient of
# this shape stays on the two-launch form)
@pytest.mark.parametrize("dy_e5m2", [False, True])
@pytest.mark.parametrize("shape", [(8208, 2048, 2064), (16400, 2064, 4112), (1040, 4112, 4112)])
def test_fused_cast_against_oracle_and_two_launch_form(shape, dy_e5m2):
    M, K, N = shape
    print("fused cast", shape, "e5m2" if dy_e5m2 else "e4m3", flush=True)
    x, w, dy = synth.fp8_linear_inputs(3, 0, M=M, K=K, N=N)
    xd, wd, dyd = to_dev_bf16(x), to_dev_bf16(w), to_dev_bf16(dy)
    fused = run_step(xd, wd, dyd, M, K, N, True, dy_e5m2)
    plain = run_step(xd, wd, dyd, M, K, N, False, dy_e5m2)
    assert tw.tweo_fused_cast_timeouts() == 0
    want = []
    for t, e5 in ((x, False), (w, False), (dy, dy_e5m2)):
        amax = oracle.amax_bf16(t)
        s, si = oracle.scale_from_amax_e5m2(amax) if e5 else oracle.scale_from_amax(amax)
        q, qT = oracle.quantize_e5m2(t, s) if e5 else oracle.quantize_e4m3(t, s)
        want.append((q, qT, amax, s, si))
    for i, (q, qT, amax, s, si) in enumerate(want):
        assert np.array_equal(fused[0][2 * i], q), ("codes", i)
        assert np.array_equal(fused[0][2 * i + 1], qT), ("transposed codes", i)
        got = fused[1][3 * i:3 * i + 3].view(np.uint32)
        assert np.array_equal(got, np.array([amax, s, si], np.float32).view(np.uint32)), ("scalars", i)
    # the two forms of the entry points: the same bytes everywhere, GEMM outputs and penalty included
    for a, b in zip(fused[0], plain[0]):
        assert np.array_equal(a, b)
    assert np.array_equal(fused[1].view(np.uint32), plain[1].view(np.uint32))
    for a, b in zip(fused[2], plain[2]):
        assert np.array_equal(a, b)
    assert fused[3] == plain[3]


def test_fused_cast_degenerate_tensors():
    # a NaN poisons the amax (scale 1, as everywhere else); an all-zero tensor has amax 0, scale 1
    M, K, N = 8208, 2048, 2064
    x, w, dy = synth.fp8_linear_inputs(1, 0, M=M, K=K, N=N)
    x = x.copy()
    x[M - 1, K - 1] = 0x7FC0
    dy = np.zeros_like(dy)
    fused = run_step(to_dev_bf16(x), to_dev_bf16(w), to_dev_bf16(dy), M, K, N, True, False)
    plain = run_step(to_dev_bf16(x), to_dev_bf16(w), to_dev_bf16(dy), M, K, N, False, False)
    sc = fused[1]
    assert np.isnan(sc[0]) and sc[1] == 1.0 and sc[2] == 1.0
    assert sc[6] == 0.0 and sc[7] == 1.0 and sc[8] == 1.0
    assert not fused[0][4].any() and not fused[0][5].any()
    for a, b in zip(fused[0], plain[0]):
        assert np.array_equal(a, b)
    assert np.array_equal(fused[1].view(np.uint32), plain[1].view(np.uint32))
    assert tw.tweo_fused_cast_timeouts() == 0


def test_fused_cast_is_skipped_under_capture_and_when_switched_off():
    # a captured graph must replay with new data: the entry point records the two-launch form
    M, K, N = 8208, 2048, 528
    x, w, _ = synth.fp8_linear_inputs(3, 0, M=M, K=K, N=N)
    xd, wd = to_dev_bf16(x), to_dev_bf16(w)
    u8 = lambda *s: torch.full(s, 0x55, dtype=torch.uint8, device=DEV)
    xq, xqT, wq, wqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N)
    sc = torch.zeros(16, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD_BF16, M, N, K)
    tw.tweo_fp8_linear_fwd_bf16(xd, wd, y, saved, workspace=ws)
    torch.cuda.synchronize()
    eager = (xq.cpu().numpy().copy(), bf16_bits(y).copy())
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            tw.tweo_fp8_linear_fwd_bf16(xd, wd, y, saved, workspace=ws)
    for rep in range(3):
        if rep == 1:
            xd.mul_(2.0)   # new data between replays: amax and codes must follow it
        y.zero_()
        xq.fill_(0x55)
        graph.replay()
        torch.cuda.synchronize()
        if rep == 0:
            assert np.array_equal(xq.cpu().numpy(), eager[0]) and np.array_equal(bf16_bits(y), eager[1])
        else:
            assert float(sc[0]) == 2.0 * oracle.amax_bf16(x)
            assert np.array_equal(xq.cpu().numpy(), eager[0])  # scale halves as the data doubles
    assert tw.tweo_fused_cast_timeouts() == 0


@pytest.mark.parametrize("e5m2", [False, True])
@pytest.mark.parametrize("shape", [(4112, 4112), (272, 1040), (16, 16)])
def test_amax_quantize_in_one_call(shape, e5m2):
    # the stand-alone entry point: one launch from 2^24 elements, two below; oracle bits either way
    rows, cols = shape
    print("amax_quantize_f8", shape, "e5m2" if e5m2 else "e4m3", flush=True)
    x = synth.fp8_linear_inputs(3, 2, M=rows, K=cols, N=16)[0]
    q = torch.full((rows, cols), 0x55, dtype=torch.uint8, device=DEV)
    qT = torch.full((cols, rows), 0x55, dtype=torch.uint8, device=DEV)
    sc = torch.full((12,), -3.0, dtype=torch.float32, device=DEV)
    ws = torch.full((4096,), 0xA5, dtype=torch.uint8, device=DEV)
    tw.tweo_amax_quantize_f8(to_dev_bf16(x), sc[0:1], q, qT, sc[4:5], sc[8:9], ws, e5m2=e5m2)
    torch.cuda.synchronize()
    amax = oracle.amax_bf16(x)
    s, si = oracle.scale_from_amax_e5m2(amax) if e5m2 else oracle.scale_from_amax(amax)
    oq, oqT = oracle.quantize_e5m2(x, s) if e5m2 else oracle.quantize_e4m3(x, s)
    assert np.array_equal(q.cpu().numpy(), oq) and np.array_equal(qT.cpu().numpy(), oqT)
    got = sc.cpu().numpy()[[0, 4, 8]].view(np.uint32)
    assert np.array_equal(got, np.array([amax, s, si], np.float32).view(np.uint32))
    assert tw.tweo_fused_cast_timeouts() == 0


def test_every_call_takes_its_own_maxima():
    # Calls in a row on one workspace whose second tensor's maximum changes from call to call
    # (forwards with weights w and 4 w in turn; the gradient of this shape is small and takes the
    # two-launch form, whose workgroup maxima land in the same words in between).  The workgroups exchange their maxima through words that earlier calls also wrote:
    # a word of an earlier call taken for this call's would cast a part of the weight with another
    # call's scale.  Codes and scalars of every call against the two-launch form (itself checked
    # against the oracle).
    M, K, N = 8192, 2048, 256   # 2^24 activation elements: the one-launch form; a small weight and gradient
    x, w, dy = synth.fp8_linear_inputs(3, 0, M=M, K=K, N=N)
    w4 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(w) * np.float32(4.0))
    xd, dyd = to_dev_bf16(x), to_dev_bf16(dy)
    wds = [to_dev_bf16(w), to_dev_bf16(w4)]
    u8 = lambda *s: torch.full(s, 0x55, dtype=torch.uint8, device=DEV)
    xq, xqT, wq, wqT, dyq, dyqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N), u8(M, N), u8(N, M)
    sc = torch.zeros(16, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    dw = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD_BF16, M, N, K)
    wsb = workspace(tw.TWEO_OP_FP8_LINEAR_BWD_BF16, M, N, K)
    ws = ws if ws.numel() >= wsb.numel() else wsb   # one workspace for both calls

    def step(wd):
        tw.tweo_fp8_linear_fwd_bf16(xd, wd, y, saved, workspace=ws)
        tw.tweo_fp8_linear_bwd_bf16(dyd, saved, K, dyq, dyqT, dx, dw, ws)

    want = []
    tw.tweo_set_fused_cast(False)
    try:
        for i, wd in enumerate(wds):
            step(wd)
            torch.cuda.synchronize()
            want.append([t.clone() for t in (wq, wqT, xq, dyq, sc)])
            amax = oracle.amax_bf16(w if i == 0 else w4)
            s, _ = oracle.scale_from_amax(amax)
            assert np.array_equal(wq.cpu().numpy(), oracle.quantize_e4m3(w if i == 0 else w4, s)[0])
    finally:
        tw.tweo_set_fused_cast(True)
    bad = torch.zeros((), dtype=torch.int64, device=DEV)
    for it in range(300):
        step(wds[it & 1])
        for got, ref in zip((wq, wqT, xq, dyq, sc), want[it & 1]):
            bad += (got != ref).any()
    assert int(bad) == 0, "%d tensors of 1500 differ from the two-launch form" % int(bad)
    assert tw.tweo_fused_cast_timeouts() == 0
