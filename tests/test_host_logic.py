"""Host-side logic of the C-ABI library that needs no GPU: workspace sizing and the argument checks
that return before anything is launched (the pointers below are never dereferenced)."""
import ctypes

import numpy as np
import pytest

import paper_2511_23225_amd as tw

OPS = (tw.TWEO_OP_FP8_LINEAR_FWD, tw.TWEO_OP_FP8_LINEAR_BWD, tw.TWEO_OP_W8A8_LINEAR,
       tw.TWEO_OP_FP8_LINEAR_FWD_BF16, tw.TWEO_OP_FP8_LINEAR_BWD_BF16)
SHAPES = [(256, 512, 512), (8192, 768, 2304), (50432, 2304, 768), (50432, 768, 3072), (16384, 6144, 2048),
          (16384, 2048, 2048), (16, 12288, 4096), (200, 392, 512)]


def test_workspace_sizes():
    for M, N, K in SHAPES:
        sizes = [tw.tweo_workspace_bytes(op, M, N, K) for op in OPS]
        assert all(s > 0 and s % 256 == 0 for s in sizes), (M, N, K, sizes)
        fwd, bwd, _, fwd_bf16, bwd_bf16 = sizes
        # the bf16 entry points put 4 KB of amax partials in front of the plain operation's workspace
        assert fwd_bf16 == fwd + 4096 and bwd_bf16 == bwd + 4096
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_FWD, 0, 5, 5) == 256  # nonsense sizes: the minimum
    assert tw.tweo_workspace_bytes(99, 256, 256, 256) == 256                    # unknown operation


def test_k_split_scratch_is_in_the_backward_workspace():
    # weight gradient [N,K] over M tokens: 2304x768 = 27 tiles of 256x256 under a contraction of
    # 50432 -> 9 runs of fp32 sums on a 256-CU device (the CU count falls back to 256 without a GPU)
    M, N, K = 50432, 2304, 768
    bwd = tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, M, N, K)
    assert bwd == 256 + 9 * N * K * 4
    # the LLaMA output projection: 64 tiles, 4 runs; a contraction of 8192 gives 4 runs of 16 stages
    # for up to 42 tiles and none for 64; one of 4096 is not split
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, 16384, 2048, 2048) == 256 + 4 * 2048 * 2048 * 4
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, 8192, 2304, 768) == 256 + 4 * 2304 * 768 * 4
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, 8192, 4096, 1024) == 512
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, 4096, 768, 768) == 512
    # many tiles: nothing beyond the fixed part
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_FP8_LINEAR_BWD, 16384, 6144, 2048) == 512


def test_argument_checks_return_before_any_launch():
    L = tw.load()
    buf = np.zeros(1 << 16, np.uint8)
    base = buf.ctypes.data + (-buf.ctypes.data) % 16
    p = lambda off=0: ctypes.c_void_p(base + off)
    INV, UNS, WSP = tw.TWEO_ERR_INVALID_ARG, tw.TWEO_ERR_UNSUPPORTED, tw.TWEO_ERR_WORKSPACE
    # null and misaligned pointers
    assert L.tweo_amax(None, 64, p(), None) == INV
    assert L.tweo_amax(p(2), 64, p(), None) == INV
    assert L.tweo_quantize_e4m3(p(), 16, 16, None, p(), p(), None, None, None) == INV
    assert L.tweo_quantize_e5m2(p(), 16, 12, p(), p(), p(), None, None, None) == UNS      # cols % 8
    assert L.tweo_amax_quantize_f8(p(), 16, 16, 0, p(), p(), None, p(), p(), p(), 4096, None) == INV   # no qT
    assert L.tweo_amax_quantize_f8(p(), 16, 24, 0, p(), p(), p(), p(), p(), p(), 4096, None) == UNS   # cols % 16
    assert L.tweo_amax_quantize_f8(p(), 16, 16, 0, p(), p(), p(), p(), p(), p(), 4095, None) == WSP   # workspace
    assert L.tweo_fused_cast_timeouts(None) == INV
    assert L.tweo_quantize_i8(p(), 12, 1.0, p(), None) == UNS                             # n % 8
    assert L.tweo_quantize_i8(p(), 16, float("nan"), p(), None) == INV
    assert L.tweo_quantize_i8_rows(p(), 4, 16, -1.0, p(), p(), None) == INV               # eps < 0
    assert L.tweo_quantize_i8_rows(p(), 4, 12, 0.0, p(), p(), None) == UNS
    assert L.tweo_quantize_i8_rows(p(), 0, 16, 0.0, p(), p(), None) == INV
    # W8A8: shape rules, granularity flags, NaN output step
    assert L.tweo_w8a8_linear(p(), p(), 16, 16, 24, 1.0, p(), None, 0, None) == UNS       # K % 16
    assert L.tweo_w8a8_linear_scaled(p(), p(), 16, 16, 32, p(), 2, p(), 0, p(), None) == INV
    assert L.tweo_w8a8_linear_scaled(p(), p(), 16, 12, 32, p(), 1, p(), 1, p(), None) == UNS  # N % 8
    assert L.tweo_w8a8_linear_scaled_i8out(p(), p(), 16, 16, 32, p(), 1, p(), 1, float("nan"), p(), None) == INV
    # FP8 linear: penalty configuration and workspace
    pen = tw.binding.PenaltyCfg(3.0, 1e-6, 4)
    bad = tw.binding.PenaltyCfg(-1.0, 1e-6, 4)
    S = p(1024)
    assert L.tweo_fp8_linear_fwd(p(), p(), p(), p(), None, 256, 256, 256, p(), ctypes.byref(bad), S, p(), 1 << 15,
                                 None) == INV
    assert L.tweo_fp8_linear_fwd(p(), p(), p(), p(), None, 256, 256, 256, p(), ctypes.byref(pen), S, None, 0,
                                 None) == WSP
    assert L.tweo_fp8_linear_fwd(p(), p(), p(), p(), None, 256, 250, 256, p(), None, None, None, 0, None) == UNS
    assert L.tweo_fp8_linear_bwd(p(), p(), p(), p(), p(), p(), p(), 250, 256, 256, p(), p(), None, 0, None) == UNS
    assert L.tweo_fp8_linear_bwd_bf16(p(), None, 256, 256, 256, p(), p(), p(), p(), p(), 8192, None) == INV
    assert L.tweo_set_gemm_tile(99) == INV and L.tweo_set_gemm_tile(0) == tw.TWEO_OK
    for code in range(5):
        assert tw.status_string(code)


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
