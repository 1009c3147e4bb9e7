"""GPU parity of the FP8 linear forward (+ fused TWEO penalty) and backward, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import (DEV, PEN, to_dev_bf16, to_dev, bf16_bits, scalar_f32, gpu_amax, gpu_quantize,
                      workspace, check_gemm, check_penalty)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def oracle_quantized(x):
    amax = oracle.amax_bf16(x)
    s, si = oracle.scale_from_amax(amax)
    q, qT = oracle.quantize_e4m3(x, s)
    return q, qT, si


def run_fwd(xq, wq, sxi, swi, M, N, K, residual=None, pen=PEN):
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD, M, N, K)
    tw.tweo_fp8_linear_fwd(to_dev(xq), scalar_f32(sxi), to_dev(wq), scalar_f32(swi), y,
                           residual_bf16=None if residual is None else to_dev_bf16(residual),
                           pen=pen, penalty_sum=S if pen else None, workspace=ws)
    torch.cuda.synchronize()
    return bf16_bits(y), float(S.cpu()[0])


CASES = [  # (cfg, gemm, M, K, N): several tiles and ragged tails in M and N
    (0, 0, 256, 512, 512),
    (0, 0, 200, 384, 136),
    (1, 0, 515, 768, 264),
    (2, 0, 333, 256, 1000),
    (3, 4, 130, 1408, 72),
    (0, 0, 16, 16, 8),
    (3, 0, 777, 256, 520),
]


@pytest.mark.parametrize("tile", [0, 1, 3, 4, 6, 8, 11, 13, 14])
@pytest.mark.parametrize("case", CASES)
def test_fwd_with_penalty(case, tile):
    cfg, gi, M, K, N = case
    say("fwd cfg=%d gemm=%d M=%d K=%d N=%d tile=%d" % (cfg, gi, M, K, N, tile))
    x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi)
    tw.tweo_set_gemm_tile(tile)
    try:
        got, S = run_fwd(xq, wq, sxi, swi, M, N, K)
    finally:
        tw.tweo_set_gemm_tile(0)
    check_gemm(got, ref, refabs, K, "fwd")
    Sref = oracle.penalty_sum(refbf, *PEN)
    # the 256x512x512 workload meets the plain 1e-4 bar; the ragged tile-coverage cases are tiny
    check_penalty(S, got, refbf, Sref, PEN, strict=(M, K, N) == (256, 512, 512))


# shapes the deferred-epilogue kernel (variant 15) takes: whole 256x256 tiles; a tile is written
# out over the first 3 (K < 1024), 7 (K < 2048) or 15 stages of its successor; 272 and 544 tiles
# give workgroups 2 and 3 tiles on a 256-CU machine, i.e. first tile, tiles written out under
# their successor, and last tile
DEFER_CASES = [
    (0, 0, 512, 1024, 768),
    (1, 0, 1024, 512, 512),
    (3, 0, 4352, 1024, 4096),
    (3, 1, 8192, 1152, 4352),
    (2, 0, 4352, 640, 4096),
    (3, 0, 4352, 2048, 8192),
    (3, 2, 8192, 2304, 4352),
]


@pytest.mark.parametrize("case", DEFER_CASES)
def test_fwd_deferred_epilogue_kernel(case):
    cfg, gi, M, K, N = case
    say("fwd deferred cfg=%d gemm=%d M=%d K=%d N=%d" % (cfg, gi, M, K, N))
    x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi)
    outs = []
    for pen in (PEN, None):
        tw.tweo_set_gemm_tile(15)
        try:
            got, S = run_fwd(xq, wq, sxi, swi, M, N, K, pen=pen)
        finally:
            tw.tweo_set_gemm_tile(0)
        check_gemm(got, ref, refabs, K, "fwd")
        if pen:
            Sref = oracle.penalty_sum(refbf, *PEN)
            check_penalty(S, got, refbf, Sref, PEN, strict=M * N >= 1 << 20)
        outs.append(got)
    assert np.array_equal(outs[0], outs[1])  # the penalty does not change the stored output


# the 192x256 flavour of the deferred-epilogue kernel (variant 16): any M (rows past M in the last
# row of tiles are loaded as copies, never stored or penalised), K >= 2048; 22 x 12 = 264 tiles
# give some workgroups a second tile
DEFER192_CASES = [
    (3, 0, 448, 2048, 512),
    (3, 1, 4160, 2048, 3072),
    (2, 0, 1000 // 8 * 8, 2304, 256),
]


@pytest.mark.parametrize("case", DEFER192_CASES)
def test_fwd_deferred_epilogue_kernel_192(case):
    cfg, gi, M, K, N = case
    say("fwd deferred 192 cfg=%d gemm=%d M=%d K=%d N=%d" % (cfg, gi, M, K, N))
    x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi)
    for pen in (PEN, None):
        tw.tweo_set_gemm_tile(16)
        try:
            got, S = run_fwd(xq, wq, sxi, swi, M, N, K, pen=pen)
        finally:
            tw.tweo_set_gemm_tile(0)
        check_gemm(got, ref, refabs, K, "fwd")
        if pen:
            Sref = oracle.penalty_sum(refbf, *PEN)
            check_penalty(S, got, refbf, Sref, PEN, strict=M * N >= 1 << 20)


@pytest.mark.parametrize("shape", [(16384, 2048, 6144, 15), (16384, 5632, 2048, 15), (8192, 768, 3072, 15),
                                   (4096, 512, 16384, 15), (6144, 16384, 2048, 16), (5632, 16384, 2048, 16),
                                   (2048, 16384, 5632, 16), (12352, 2048, 4096, 16)])
def test_fwd_deferred_kernel_matches_streaming_kernel_bitwise(shape):
    # Both kernels add a block's K slabs in the same order with the same MFMA, so their outputs
    # are the same bits; at these sizes every workgroup owns several tiles (first tile, tiles
    # written out under their successor, last tile), twice over to catch anything left behind
    M, K, N, variant = shape
    say("fwd deferred (variant %d) vs streaming M=%d K=%d N=%d" % (variant, M, K, N))
    g = torch.Generator(device=DEV)
    g.manual_seed(M + 3 * K + 7 * N)
    xq = torch.randint(0, 0x78, (M, K), dtype=torch.uint8, device=DEV, generator=g)
    wq = torch.randint(0, 0x78, (N, K), dtype=torch.uint8, device=DEV, generator=g)
    xq |= torch.randint(0, 2, (M, K), dtype=torch.uint8, device=DEV, generator=g) << 7
    sc = scalar_f32(0.01)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD, M, N, K)
    outs, sums = [], []
    for tile in (11, variant, variant):
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)
        S = torch.zeros(2, dtype=torch.float64, device=DEV)
        tw.tweo_set_gemm_tile(tile)
        try:
            tw.tweo_fp8_linear_fwd(xq, sc, wq, sc, y, pen=PEN, penalty_sum=S, workspace=ws)
            torch.cuda.synchronize()
        finally:
            tw.tweo_set_gemm_tile(0)
        outs.append(y.view(torch.int16))
        sums.append(float(S.cpu()[0]))
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert abs(sums[1] - sums[0]) <= 1e-5 * abs(sums[0]) and sums[1] == sums[2]


@pytest.mark.parametrize("with_residual", [False, True])
def test_fwd_stream_k_split_of_the_last_round(with_residual):
    # 64 tiles of 256x256 and a long K on a 256-CU machine: the K loop of every tile is cut over
    # four workgroups, partial accumulators go through the workspace, the last arrival adds them
    # in K order and runs the epilogue (scale, residual, bf16, penalty).  Checked on every
    # element, against the plain schedule, and for run-to-run identity.
    cfg, gi, M, K, N = 3, 0, 2048, 8192, 2048
    say("fwd stream-K M=%d K=%d N=%d residual=%s" % (M, K, N, with_residual))
    x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    res = synth.residual_input(cfg, gi, M, N) if with_residual else None
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, residual=res)
    Sref = oracle.penalty_sum(refbf, *PEN)
    runs = []
    for on in (True, True, False):
        tw.tweo_set_stream_k(on)
        try:
            got, S = run_fwd(xq, wq, sxi, swi, M, N, K, residual=res)
        finally:
            tw.tweo_set_stream_k(False)
        check_gemm(got, ref, refabs, K, "fwd stream-K=%s" % on)
        check_penalty(S, got, refbf, Sref, PEN, strict=True)
        runs.append((got, S))
    assert np.array_equal(runs[0][0], runs[1][0]) and runs[0][1] == runs[1][1]  # deterministic


def test_fwd_residual_is_block_output():
    # y = x + f(x): the penalised tensor is the block output (Sec. 3.3)
    cfg, gi, M, K, N = 1, 3, 384, 1024, 256
    say("fwd residual M=%d K=%d N=%d" % (M, K, N))
    x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    res = synth.residual_input(cfg, gi, M, N)
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, residual=res)
    got, S = run_fwd(xq, wq, sxi, swi, M, N, K, residual=res)
    check_gemm(got, ref, refabs, K, "fwd+residual")
    Sref = oracle.penalty_sum(refbf, *PEN)
    check_penalty(S, got, refbf, Sref, PEN, strict=False)
    got2, _ = run_fwd(xq, wq, sxi, swi, M, N, K, residual=res, pen=None)
    assert np.array_equal(got, got2)  # the penalty does not change the stored output


@pytest.mark.parametrize("pen", [(3.0, 1e-6, 4), (2.0, 1e-6, 4), (5.0, 1e-6, 4), (5.0, 0.0, 2),
                                 (3.0, 1e-6, 3), (4.0, 1e-6, 6)])
def test_penalty_hyperparameters(pen):
    M, K, N = 256, 512, 512
    say("penalty", pen)
    x, w, _ = synth.fp8_linear_inputs(0, 0)
    xq, _, sxi = oracle_quantized(x)
    wq, _, swi = oracle_quantized(w)
    _, _, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, want_abs=False)
    got, S = run_fwd(xq, wq, sxi, swi, M, N, K, pen=pen)
    Sref = oracle.penalty_sum(refbf, *pen)
    # p = 4 (the paper's setting) meets the 1e-4 bar.  For larger p the sum is carried by a
    # handful of elements, and a stored value that differs from the oracle's by one bf16 ulp
    # (fp32 vs fp64 arithmetic in front of the rounding) moves its term by p * 2^-8.
    tol = 1e-4 if pen[2] <= 4 else 1e-3
    assert abs(S - Sref) <= tol * Sref, (S, Sref)
    # consistency of the fused reduction with the tensor the kernel stored (not a parity claim)
    y = synth.bf16_bits_to_f32(got).astype(np.float64)
    S_self = np.sum((np.abs(y) / (pen[0] + pen[1])) ** pen[2])
    assert abs(S - S_self) <= 2e-6 * S_self, (S, S_self)


def test_penalty_printed_regimes_through_the_gemm():
    # W = c*I makes every output magnitude known: |y| = 0.5 tau, tau, 10 tau -> mean 0.0625, 1, 1e4
    M = N = K = 128
    for ratio, printed in ((0.5, 0.0625), (1.0, 1.0), (10.0, 10000.0)):
        say("penalty regime", ratio)
        # decoded operands: x = 1.5 everywhere on the diagonal selector, w = diag
        xq = np.full((M, K), oracle.e4m3_encode(1.5), np.uint8)
        wq = np.zeros((N, K), np.uint8)
        wq[np.arange(N), np.arange(N)] = oracle.e4m3_encode(2.0)
        # y = 1.5 * 2 * sxi * swi = 3 * ratio  with sxi*swi = ratio (powers of two / exact)
        got, S = run_fwd(xq, wq, np.float32(ratio), np.float32(1.0), M, N, K, pen=(3.0, 0.0, 4))
        y = synth.bf16_bits_to_f32(got)
        assert np.all(y == np.float32(3.0 * ratio))
        assert abs(S / (M * N) - printed) <= 1e-6 * printed


@pytest.mark.parametrize("tile", [0, 1, 3, 4, 6, 8, 11, 13, 14, 15])
@pytest.mark.parametrize("case", [(0, 0, 256, 512, 512), (1, 1, 208, 256, 144), (3, 0, 144, 640, 400),
                                  (3, 0, 1024, 512, 768)])
def test_bwd(case, tile):
    cfg, gi, M, K, N = case
    say("bwd cfg=%d M=%d K=%d N=%d tile=%d" % (cfg, M, K, N, tile))
    x, w, dy = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    xq, xqT, sxi = oracle_quantized(x)
    wq, wqT, swi = oracle_quantized(w)
    dyq, dyqT, sdyi = oracle_quantized(dy)
    dx_ref, dx_abs = oracle.fp8_linear_dgrad(dyq, wq, sdyi, swi)
    dw_ref, dw_abs = oracle.fp8_linear_wgrad(dyq, xq, sdyi, sxi)
    dx = torch.full((M, K), float('nan'), dtype=torch.bfloat16, device=DEV)
    dw = torch.full((N, K), float('nan'), dtype=torch.bfloat16, device=DEV)
    tw.tweo_set_gemm_tile(tile)
    try:
        tw.tweo_fp8_linear_bwd(to_dev(dyq), to_dev(dyqT), scalar_f32(sdyi), to_dev(wqT),
                               scalar_f32(swi), to_dev(xqT), scalar_f32(sxi), M, N, K, dx, dw,
                               workspace(tw.TWEO_OP_FP8_LINEAR_BWD, M, N, K))
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    check_gemm(bf16_bits(dx), dx_ref, dx_abs, N, "dgrad")
    check_gemm(bf16_bits(dw), dw_ref, dw_abs, M, "wgrad")


# outputs of a few 256x256 tiles under a very long contraction: the K split (several workgroups per
# tile, fp32 runs added in order by a second kernel).  wgrad over 16384 tokens of a 768-wide layer
# (8 runs on the deferred-epilogue kernel), a ragged one whose last K stage is partial (the
# register-staged kernel), a dgrad over a long N, a wgrad over 8192 tokens (4 runs of 16 stages) and
# one whose stages do not divide evenly over the runs (67 stages, 4 runs), and one with 48 tiles
# under 80 stages (5 runs: from 80 stages on, up to half as many tiles as CUs are split); each run twice.
@pytest.mark.parametrize("case", [(1, 1, 16384, 768, 768), (3, 0, 16400, 264, 528), (0, 0, 256, 512, 16384),
                                  (1, 0, 8192, 768, 2304), (1, 2, 8576, 512, 768), (3, 0, 10240, 2048, 1536)])
def test_bwd_k_split(case):
    cfg, gi, M, K, N = case
    say("bwd K split cfg=%d M=%d K=%d N=%d" % (cfg, M, K, N))
    x, w, dy = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
    xq, xqT, sxi = oracle_quantized(x)
    wq, wqT, swi = oracle_quantized(w)
    dyq, dyqT, sdyi = oracle_quantized(dy)
    dx_ref, dx_abs = oracle.fp8_linear_dgrad(dyq, wq, sdyi, swi)
    dw_ref, dw_abs = oracle.fp8_linear_wgrad(dyq, xq, sdyi, sxi)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_BWD, M, N, K)
    assert ws.numel() >= 2 * 4 * min(M * K, N * K)  # the query asks for the runs' scratch
    outs = []
    for rep in range(2):
        dx = torch.full((M, K), float('nan'), dtype=torch.bfloat16, device=DEV)
        dw = torch.full((N, K), float('nan'), dtype=torch.bfloat16, device=DEV)
        ws.fill_(0xFF)  # the scratch needs no initialisation: poison it
        tw.tweo_fp8_linear_bwd(to_dev(dyq), to_dev(dyqT), scalar_f32(sdyi), to_dev(wqT),
                               scalar_f32(swi), to_dev(xqT), scalar_f32(sxi), M, N, K, dx, dw, ws)
        torch.cuda.synchronize()
        outs.append((bf16_bits(dx), bf16_bits(dw)))
    check_gemm(outs[0][0], dx_ref, dx_abs, N, "dgrad")
    check_gemm(outs[0][1], dw_ref, dw_abs, M, "wgrad")
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])  # run to run
    # without the scratch the plain schedule runs: same result within the same bounds
    dw = torch.full((N, K), float('nan'), dtype=torch.bfloat16, device=DEV)
    tw.tweo_fp8_linear_bwd(to_dev(dyq), to_dev(dyqT), scalar_f32(sdyi), to_dev(wqT), scalar_f32(swi),
                           to_dev(xqT), scalar_f32(sxi), M, N, K, None, dw, None)
    torch.cuda.synchronize()
    check_gemm(bf16_bits(dw), dw_ref, dw_abs, M, "wgrad, plain schedule")


def test_whole_path_from_bf16_and_determinism():
    cfg, gi, M, K, N = 0, 0, 256, 512, 512
    say("bf16 path M=%d K=%d N=%d" % (M, K, N))
    x, w, dy = synth.fp8_linear_inputs(cfg, gi)
    xd, wd, dyd = to_dev_bf16(x), to_dev_bf16(w), to_dev_bf16(dy)
    u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=DEV)
    outs = []
    for rep in range(2):
        xq, xqT, wq, wqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N)
        dyq, dyqT = u8(M, N), u8(N, M)
        sc = torch.full((16,), -3.0, dtype=torch.float32, device=DEV)
        saved = tw.make_saved(xq, xqT, wq, wqT, sc)
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
        dx = torch.full((M, K), float('nan'), dtype=torch.bfloat16, device=DEV)
        dw = torch.full((N, K), float('nan'), dtype=torch.bfloat16, device=DEV)
        S = torch.zeros(2, dtype=torch.float64, device=DEV)
        ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD_BF16, M, N, K)
        tw.tweo_fp8_linear_fwd_bf16(xd, wd, y, saved, pen=PEN, penalty_sum=S, workspace=ws)
        tw.tweo_fp8_linear_bwd_bf16(dyd, saved, K, dyq, dyqT, dx, dw, ws)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy().copy() for t in (xq, xqT, wq, wqT, dyq, dyqT)] +
                    [bf16_bits(y), bf16_bits(dx), bf16_bits(dw), S.cpu().numpy().copy(),
                     sc.cpu().numpy().copy()])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)  # run-to-run identical, penalty included
    gxq, gxqT, gwq, gwqT, gdyq, gdyqT, gy, gdx, gdw, gS, gsc = outs[0]
    oxq, oxqT, sxi = oracle_quantized(x)
    owq, owqT, swi = oracle_quantized(w)
    odyq, odyqT, sdyi = oracle_quantized(dy)
    for g, o in ((gxq, oxq), (gxqT, oxqT), (gwq, owq), (gwqT, owqT), (gdyq, odyq), (gdyqT, odyqT)):
        assert np.array_equal(g, o)
    want_sc = [oracle.amax_bf16(x), *oracle.scale_from_amax(oracle.amax_bf16(x)),
               oracle.amax_bf16(w), *oracle.scale_from_amax(oracle.amax_bf16(w)),
               oracle.amax_bf16(dy), *oracle.scale_from_amax(oracle.amax_bf16(dy))]
    assert np.array_equal(gsc[:9], np.array(want_sc, np.float32))
    ref, refabs, refbf = oracle.fp8_linear_fwd(oxq, owq, sxi, swi)
    check_gemm(gy, ref, refabs, K, "fwd")
    Sref = oracle.penalty_sum(refbf, *PEN)
    assert abs(gS[0] - Sref) <= 1e-4 * Sref
    dx_ref, dx_abs = oracle.fp8_linear_dgrad(odyq, owq, sdyi, swi)
    dw_ref, dw_abs = oracle.fp8_linear_wgrad(odyq, oxq, sdyi, sxi)
    check_gemm(gdx, dx_ref, dx_abs, N, "dgrad")
    check_gemm(gdw, dw_ref, dw_abs, M, "wgrad")


@pytest.mark.parametrize("tile,M,N,K", [(4, 64, 64, 256), (15, 256, 256, 512)])
def test_mfma_sums_products_in_groups_of_8_with_a_13_bit_window(tile, M, N, K):
    # What the earned bound of check_gemm rests on.  The FP8 MFMA adds its products in groups of 8
    # consecutive k after aligning them to the group's largest product: a product of at least
    # 2^-13 of that one survives, a product of 2^-14 of it is dropped; products in OTHER groups
    # are not affected.  Row 0: k = 0, 1 hold +B*B and -B*B (they cancel exactly), k = 2..7 (same
    # group) and k = 8..13 (next group) hold six products of B*B * 2^-j each.  The fp64 oracle
    # keeps all twelve; the hardware keeps twelve for j = 13 and only the six of the other group
    # for j = 14.  Either way the difference stays inside the bound (2^-10 + K 2^-24) sum|x w|.
    enc = oracle.e4m3_encode
    for big in (1.0, 16.0):
        for j, kept in ((10, 12), (13, 12), (14, 6), (16, 6)):
            say("mfma window tile=%d big=%g j=%d" % (tile, big, j))
            a = min(j, 8)
            xs, wsml = big * 2.0 ** -a, big * 2.0 ** -(j - a)   # exact E4M3 values (powers of two)
            xq, wq = np.zeros((M, K), np.uint8), np.zeros((N, K), np.uint8)
            xq[0, 0], wq[0, 0] = enc(big), enc(big)
            xq[0, 1], wq[0, 1] = enc(-big), enc(big)
            for k in list(range(2, 8)) + list(range(8, 14)):
                xq[0, k], wq[0, k] = enc(xs), enc(wsml)
            ref, refabs, _ = oracle.fp8_linear_fwd(xq, wq, 1.0, 1.0)
            assert ref[0, 0] == 12 * big * big * 2.0 ** -j and refabs[0, 0] == ref[0, 0] + 2 * big * big
            tw.tweo_set_gemm_tile(tile)
            try:
                got, _ = run_fwd(xq, wq, np.float32(1.0), np.float32(1.0), M, N, K, pen=None)
            finally:
                tw.tweo_set_gemm_tile(0)
            y00 = float(synth.bf16_bits_to_f32(got[0:1, 0:1])[0, 0])
            assert y00 == kept * big * big * 2.0 ** -j, (big, j, y00)
            assert abs(y00 - ref[0, 0]) <= (2.0 ** -10 + K * 2.0 ** -24) * refabs[0, 0]
            assert not got[1:].any() and not got[0, 1:].any()


def test_error_paths_need_no_launch():
    y = torch.empty((16, 16), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((16, 16), dtype=torch.uint8, device=DEV)
    s = scalar_f32(1.0)
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_fp8_linear_fwd(q, s, q, s, y, pen=PEN, penalty_sum=S, workspace=None)
    assert e.value.status == tw.TWEO_ERR_WORKSPACE
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_fp8_linear_fwd(q, s, q, s, y, pen=(3.0, 1e-6, 9), penalty_sum=S,
                               workspace=workspace(0, 16, 16, 16))
    assert e.value.status == tw.TWEO_ERR_UNSUPPORTED
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_fp8_linear_fwd(q[:, :8].contiguous(), s, q[:, :8].contiguous(), s, y)
    assert e.value.status == tw.TWEO_ERR_UNSUPPORTED  # K % 16 != 0
