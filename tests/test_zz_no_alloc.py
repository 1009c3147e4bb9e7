"""The forward entry point that allocates nothing (its penalty partial sums live in a device
array inside the library) against the entry point that takes a workspace: same output bits and
the same penalty scalar, on two calls in a row, the second with a smaller input, which finds
the first call's contents in the array."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, PEN, to_dev, to_dev_bf16, bf16_bits, scalar_f32, workspace, check_gemm

pytestmark = pytest.mark.gpu


def quantized(x):
    s, si = oracle.scale_from_amax(oracle.amax_bf16(x))
    q, _ = oracle.quantize_e4m3(x, s, transpose=False)
    return q, si


@pytest.mark.parametrize("with_residual", [False, True])
def test_static_scratch_forward_matches_the_workspace_forward(with_residual):
    assert tw.tweo_static_scratch_bytes() == 1 << 20
    # first a shape whose partial sums fill a good part of the array's front, then a smaller one
    for cfg, gi, M, K, N in ((3, 0, 4352, 1024, 4096), (1, 1, 520, 256, 264)):
        print("no-alloc forward M=%d K=%d N=%d residual=%s" % (M, K, N, with_residual), flush=True)
        x, w, _ = synth.fp8_linear_inputs(cfg, gi, M=M, K=K, N=N)
        res = synth.residual_input(cfg, gi, M, N) if with_residual else None
        xq, sxi = quantized(x)
        wq, swi = quantized(w)
        xd, wd, sx, sw = to_dev(xq), to_dev(wq), scalar_f32(sxi), scalar_f32(swi)
        rd = None if res is None else to_dev_bf16(res)
        outs = []
        for static in (False, True):
            y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
            S = torch.full((2,), -1.0, dtype=torch.float64, device=DEV)
            if static:
                tw.tweo_fp8_linear_fwd_static(xd, sx, wd, sw, y, residual_bf16=rd, pen=PEN, penalty_sum=S)
            else:
                tw.tweo_fp8_linear_fwd(xd, sx, wd, sw, y, residual_bf16=rd, pen=PEN, penalty_sum=S,
                                       workspace=workspace(tw.TWEO_OP_FP8_LINEAR_FWD, M, N, K))
            torch.cuda.synchronize()
            outs.append((bf16_bits(y), float(S.cpu()[0])))
        assert np.array_equal(outs[0][0], outs[1][0])
        assert outs[0][1] == outs[1][1]
        # and both against the oracle, to the bars of the other forward tests
        ref, refabs, refbf = oracle.fp8_linear_fwd(xq, wq, sxi, swi, residual=res)
        check_gemm(outs[1][0], ref, refabs, K, "fwd (static scratch)")
        Sref = oracle.penalty_sum(refbf, *PEN)
        if M * N >= 1 << 20:
            assert abs(outs[1][1] - Sref) <= 1e-4 * Sref
    # without a penalty nothing of the array is used
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    tw.tweo_fp8_linear_fwd_static(xd, sx, wd, sw, y, residual_bf16=rd)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits(y), outs[1][0])


def test_static_scratch_forward_rejects_what_does_not_fit():
    q = torch.zeros((16, 16), dtype=torch.uint8, device=DEV)
    s = scalar_f32(1.0)
    S = torch.zeros(2, dtype=torch.float64, device=DEV)
    y = torch.empty((16, 16), dtype=torch.bfloat16, device=DEV)
    lib = tw.load()
    import ctypes
    pen = tw.binding.PenaltyCfg(3.0, 1e-6, 4)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    # 2^20 x 2^18 outputs would need 2^28 bytes of partial sums: refused before anything is launched
    st = lib.tweo_fp8_linear_fwd_static(p(q), p(s), p(q), p(s), None, 1 << 20, 1 << 18, 16, p(y), ctypes.byref(pen),
                                        p(S), None)
    assert st == tw.TWEO_ERR_UNSUPPORTED
    st = lib.tweo_fp8_linear_fwd_static(p(q), p(s), None, p(s), None, 16, 16, 16, p(y), ctypes.byref(pen), p(S), None)
    assert st == tw.TWEO_ERR_INVALID_ARG
