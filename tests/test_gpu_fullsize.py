"""GPU parity at the workloads' full sizes, in the launch configuration bench.py times
(shape heuristic, whole path from bf16 operands).  The oracle checks every amax and scale,
whole quantized tensors where that takes seconds (row samples otherwise), GEMM outputs on
sampled rows (rows are independent, so a sampled row is checked exactly as a full run
would; the sample holds both edge rows of every 256-row and every 192-row band, so every
tile row of every kernel variant is looked at), and the penalty against the oracle: on the
whole tensor for small layers, else on the sampled rows (1e-4) together with the property
that the returned scalar equals the sum over the tensor the kernel stored."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, PEN, to_dev_bf16, bf16_bits, check_gemm, penalty_terms, workspace

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def run_layer(x, w, dy, M, K, N, residual=None):
    u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=DEV)
    nan = lambda *s: torch.full(s, float("nan"), dtype=torch.bfloat16, device=DEV)
    t = dict(xq=u8(M, K), xqT=u8(K, M), wq=u8(N, K), wqT=u8(K, N), dyq=u8(M, N), dyqT=u8(N, M),
             y=nan(M, N), dx=nan(M, K), dw=nan(N, K),
             sc=torch.full((16,), -1.0, dtype=torch.float32, device=DEV),
             S=torch.zeros(2, dtype=torch.float64, device=DEV))
    saved = tw.make_saved(t["xq"], t["xqT"], t["wq"], t["wqT"], t["sc"])
    # one workspace for both directions, as bench.py sizes it (the backward one includes the
    # scratch of a K-split weight gradient where the shape calls for one)
    ws = torch.empty(max(tw.tweo_workspace_bytes(op, M, N, K) for op in
                         (tw.TWEO_OP_FP8_LINEAR_FWD_BF16, tw.TWEO_OP_FP8_LINEAR_BWD_BF16)),
                     dtype=torch.uint8, device=DEV)
    tw.tweo_fp8_linear_fwd_bf16(to_dev_bf16(x), to_dev_bf16(w), t["y"], saved,
                                residual_bf16=None if residual is None else to_dev_bf16(residual),
                                pen=PEN, penalty_sum=t["S"], workspace=ws)
    tw.tweo_fp8_linear_bwd_bf16(to_dev_bf16(dy), saved, K, t["dyq"], t["dyqT"], t["dx"], t["dw"], ws)
    torch.cuda.synchronize()
    return t


def rows_sample(n, count, seed):
    """Rows to check against the oracle: the first and the last row of every 256-row and of every
    192-row band (the two tile heights of the GEMM kernels, so that every tile row of the output
    is looked at, at both of its edges), plus `count` random rows."""
    rng = np.random.default_rng(seed)
    picks = [rng.choice(n, size=min(count, n), replace=False)]
    for band in (256, 192):
        first = np.arange(0, n, band)
        picks += [first, np.minimum(first + band - 1, n - 1)]
    return np.unique(np.concatenate(picks))


def check_quantized(name, bits, q_dev, qT_dev, scale, rows):
    """Every byte of q against the oracle; qT against the oracle's transpose on the whole tensor
    (rows is None) or on the sampled rows (= columns of qT).  Returns the oracle's q."""
    want, wantT = oracle.quantize_e4m3(bits, scale, transpose=rows is None)
    assert np.array_equal(q_dev.cpu().numpy(), want), name
    if rows is None:
        assert np.array_equal(qT_dev.cpu().numpy(), wantT), name + " (transposed)"
    else:
        idx = torch.from_numpy(rows).to(DEV)
        assert np.array_equal(qT_dev[:, idx].cpu().numpy(), want[rows].T), name + " (transposed)"
    return want


CASES = [  # (cfg, gemm index, full oracle for the forward + penalty?)
    (1, 1, True),    # GPT-2 proj 8192x768x768
    (1, 0, False),   # GPT-2 qkv 8192x768x2304
    (1, 3, False),   # GPT-2 fc2 8192x3072x768
    (2, 1, False),   # ViT fc1 50432x768x3072 (channel outliers)
    (2, 2, False),   # ViT fc2 50432x3072x768
    (3, 0, False),   # LLaMA qkv 16384x2048x6144
    (3, 1, False),   # LLaMA o 16384x2048x2048 (its weight gradient: 64 tiles, K split)
    (3, 2, False),   # LLaMA gate 16384x2048x5632: forward 1408 tiles = 5.5 rounds, weight gradient 240 tiles of 192x256
    (3, 3, False),   # LLaMA up, the same shape on its own data
    (3, 4, False),   # LLaMA down 16384x5632x2048
    (1, 2, False),   # GPT-2 fc1 8192x768x3072
    (2, 0, False, 18912),  # ViT qkv at 96 images: 18912 tokens, not a multiple of any tile height
    (2, 2, False, 18912),  # ViT fc2 likewise (long K forward, ragged rows in dgrad, ragged contraction in wgrad)
]


@pytest.mark.parametrize("case", CASES)
def test_full_size_layer(case):
    cfg, gi, full = case[:3]
    g = synth.CONFIGS[cfg]["gemms"][gi]
    M, K, N = (case[3] if len(case) > 3 else g.M), g.K, g.N
    say("full size cfg=%d %s M=%d K=%d N=%d" % (cfg, g.name, M, K, N))
    x, w, dy = synth.fp8_linear_inputs(cfg, gi, M=M)
    residual = synth.residual_input(cfg, gi, M, N) if g.name in ("fc2", "down", "proj") else None
    t = run_layer(x, w, dy, M, K, N, residual)
    say("  gpu done")
    sc = t["sc"].cpu().numpy()
    # amax and scales: exact, on the whole tensors
    want_sc = []
    for bits in (x, w, dy):
        a = oracle.amax_bf16(bits)
        want_sc += [a, *oracle.scale_from_amax(a)]
    assert np.array_equal(sc[:9], np.array(want_sc, np.float32))
    sx, sxi, sw, swi, sdy, sdyi = want_sc[1], want_sc[2], want_sc[4], want_sc[5], want_sc[7], want_sc[8]
    # quantized bytes: W whole; X whole when it is small, else sampled rows; dY sampled rows
    rm = rows_sample(M, 32, 11 * cfg + gi)
    wq = check_quantized("wq", w, t["wq"], t["wqT"], sw, None)
    xq = check_quantized("xq", x, t["xq"], t["xqT"], sx, rm)
    dyq = check_quantized("dyq", dy, t["dyq"], t["dyqT"], sdy, rm)
    say("  quantized bytes ok (%d sampled rows)" % rm.size)
    rs = rm
    # forward on sampled rows (or all rows)
    if full:
        ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, residual=residual)
        check_gemm(bf16_bits(t["y"]), ref, refabs, K, "fwd")
        Sref = oracle.penalty_sum(refbf, *PEN)
        S = float(t["S"].cpu()[0])
        assert abs(S - Sref) <= 1e-4 * Sref, (S, Sref)
    else:
        ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, residual=residual, rows=rs)
        got = bf16_bits(t["y"][torch.from_numpy(rs).to(DEV)])
        check_gemm(got, ref, refabs, K, "fwd rows")
        # penalty against the oracle on the sampled rows (Sec. 3.3): the sum over the rows the GPU
        # stored against the oracle's sum over its own rows, at the 1e-4 bar
        S_rows = penalty_terms(got, PEN).sum()
        S_rows_ref = oracle.penalty_sum(refbf, *PEN)
        assert abs(S_rows - S_rows_ref) <= 1e-4 * S_rows_ref, (S_rows, S_rows_ref)
        # ... and the fused reduction equals the sum over the whole stored tensor (fp64 on the
        # device copy, chunked): together the two tie the returned scalar to the oracle
        S = float(t["S"].cpu()[0])
        S_self = 0.0
        for r0 in range(0, M, 4096):
            blk = t["y"][r0:r0 + 4096].to(torch.float64).abs() / (PEN[0] + PEN[1])
            S_self += float((blk ** PEN[2]).sum().cpu())
        assert abs(S - S_self) <= 2e-6 * S_self, (S, S_self)
    say("  fwd ok")
    # dgrad on sampled rows of M
    dx_ref, dx_abs = oracle.fp8_linear_dgrad(dyq, wq, sdyi, swi, rows=rs)
    got = bf16_bits(t["dx"][torch.from_numpy(rs).to(DEV)])
    check_gemm(got, dx_ref, dx_abs, N, "dgrad rows")
    say("  dgrad ok")
    # wgrad on sampled rows of N (the contraction runs over all of M)
    rn = rows_sample(N, 8, 7 * cfg + gi)
    dw_ref, dw_abs = oracle.fp8_linear_wgrad(dyq, xq, sdyi, sxi, rows=rn)
    got = bf16_bits(t["dw"][torch.from_numpy(rn).to(DEV)])
    check_gemm(got, dw_ref, dw_abs, M, "wgrad rows")
    say("  wgrad ok")


@pytest.mark.parametrize("M", [1, 16, 64, 4096])
@pytest.mark.parametrize("gi", [0, 1, 2, 3])  # qkv, gate, up, down; gate/up at M = 4096: 688 tiles
def test_full_size_w8a8(gi, M):
    g = synth.CONFIGS[4]["gemms"][gi]
    K, N = g.K, g.N
    say("full size w8a8 %s M=%d K=%d N=%d" % (g.name, M, K, N))
    x, w = synth.w8a8_inputs(gi, M)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    tw.tweo_quantize_i8(to_dev_bf16(x), inv_x, xq)
    wq = torch.empty((N, K), dtype=torch.int8, device=DEV)
    tw.tweo_quantize_i8(to_dev_bf16(w), inv_w, wq)  # weights: same kernel, offline
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    assert np.array_equal(xq.cpu().numpy(), oxq) and np.array_equal(wq.cpu().numpy(), owq)
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    tw.tweo_w8a8_linear(xq, wq, alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
    torch.cuda.synchronize()
    if M <= 64:
        assert np.array_equal(bf16_bits(y), oracle.w8a8_linear(oxq, owq, alpha))
    else:
        rs = rows_sample(M, 16, gi)
        want = oracle.w8a8_linear(np.ascontiguousarray(oxq[rs]), owq, alpha)
        assert np.array_equal(bf16_bits(y[torch.from_numpy(rs).to(DEV)]), want)


@pytest.mark.parametrize("M", [16, 64, 4096])
@pytest.mark.parametrize("gi", [0, 3])  # qkv 4096 -> 12288 and down 11008 -> 4096
def test_full_size_w8a8_finer_granularities(gi, M):
    # W8(C)A8(K) at the 7B shapes: per-token quantisation on the GPU (all bytes and steps compared),
    # per-channel weights, bf16 and INT8 outputs (all rows for M <= 64, sampled rows for M = 4096)
    g = synth.CONFIGS[4]["gemms"][gi]
    K, N = g.K, g.N
    say("full size w8a8 W(C)A(K) %s M=%d K=%d N=%d" % (g.name, M, K, N))
    x, w = synth.w8a8_inputs(gi, M)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    wq = torch.empty((N, K), dtype=torch.int8, device=DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=DEV)
    sw = torch.empty((N,), dtype=torch.float32, device=DEV)
    tw.tweo_quantize_i8_rows(to_dev_bf16(x), 1e-6, xq, sx)
    tw.tweo_quantize_i8_rows(to_dev_bf16(w), 1e-6, wq, sw)
    oxq, osx = oracle.quantize_i8_rows(x, 1e-6)
    owq, osw = oracle.quantize_i8_rows(w, 1e-6)
    assert np.array_equal(xq.cpu().numpy(), oxq) and np.array_equal(wq.cpu().numpy(), owq)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), osx.view(np.uint32))
    assert np.array_equal(sw.cpu().numpy().view(np.uint32), osw.view(np.uint32))
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    yq = torch.full((M, N), 99, dtype=torch.int8, device=DEV)
    inv_out = np.float32(127.0) / np.float32(2.0)  # a static output step that clips the tails
    tw.tweo_w8a8_linear_scaled(xq, wq, sx, sw, y)
    tw.tweo_w8a8_linear_scaled_i8out(xq, wq, sx, sw, inv_out, yq)
    torch.cuda.synchronize()
    rs = np.arange(M) if M <= 64 else rows_sample(M, 16, gi)
    sel = torch.from_numpy(rs).to(DEV)
    want = oracle.w8a8_linear_scaled(np.ascontiguousarray(oxq[rs]), owq, np.ascontiguousarray(osx[rs]), osw)
    want_q = oracle.w8a8_linear_scaled_i8out(np.ascontiguousarray(oxq[rs]), owq, np.ascontiguousarray(osx[rs]), osw,
                                             inv_out)
    assert np.array_equal(bf16_bits(y[sel]), want)
    assert np.array_equal(yq[sel].cpu().numpy(), want_q)
    assert 0 < np.mean(np.abs(want_q) == 127) < 0.5  # some saturate, most do not


# qkv (one-launch casts, six rounds of 256x256 tiles, 192x256 weight-gradient tiles), the output
# projection (K-split weight gradient), ViT fc2 at a token count that is no multiple of a tile
# height (partial last round, ragged last band)
@pytest.mark.parametrize("shape", [(16384, 2048, 6144), (16384, 2048, 2048), (18912, 3072, 768)])
def test_full_size_step_is_deterministic_whatever_the_workspace_held(shape):
    # "Same inputs, byte-identical outputs" at the sizes bench.py times: every kernel of the step
    # that hands data from one workgroup to another (the casts' grid-wide exchange of maxima, the
    # K-split runs and their reduction, the penalty partials) does so through the workspace.  The
    # step repeated over workspaces filled with different bytes must leave the same bits in every
    # output - a word of an earlier call taken for this call's would show here.
    M, K, N = shape
    say("determinism", shape)
    x, w, dy = synth.fp8_linear_inputs(3, 0, M=M, K=K, N=N)
    xd, wd, dyd = to_dev_bf16(x), to_dev_bf16(w), to_dev_bf16(dy)
    u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=DEV)
    bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=DEV)
    xq, xqT, wq, wqT, dyq, dyqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N), u8(M, N), u8(N, M)
    y, dx, dw = bf(M, N), bf(M, K), bf(N, K)
    sc = torch.zeros(16, dtype=torch.float32, device=DEV)
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    ws = torch.empty(max(tw.tweo_workspace_bytes(op, M, N, K) for op in
                         (tw.TWEO_OP_FP8_LINEAR_FWD_BF16, tw.TWEO_OP_FP8_LINEAR_BWD_BF16)),
                     dtype=torch.uint8, device=DEV)
    outs = (xq, xqT, wq, wqT, dyq, dyqT, y.view(torch.int16), dx.view(torch.int16), dw.view(torch.int16), sc, S)
    names = ("xq", "xqT", "wq", "wqT", "dyq", "dyqT", "y", "dx", "dw", "scalars", "penalty")
    first = None
    for rep, fill in enumerate((0x00, 0xFF, 0xA5, None, None, 0x7F, None, None)):
        if fill is not None:
            ws.fill_(fill)           # None: whatever the call before left
        for t in (xq, xqT, wq, wqT, dyq, dyqT):
            t.fill_(0x55)
        for t in (y, dx, dw):
            t.fill_(float("nan"))
        tw.tweo_fp8_linear_fwd_bf16(xd, wd, y, saved, pen=PEN, penalty_sum=S, workspace=ws)
        tw.tweo_fp8_linear_bwd_bf16(dyd, saved, K, dyq, dyqT, dx, dw, ws)
        torch.cuda.synchronize()
        if first is None:
            first = [t.clone() for t in outs]
            continue
        for name, a, b in zip(names, outs, first):
            assert torch.equal(a, b), "repetition %d: %s differs in %d elements" % (rep, name, int((a != b).sum()))
    assert tw.tweo_fused_cast_timeouts() == 0
