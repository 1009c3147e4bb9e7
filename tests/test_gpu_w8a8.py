"""GPU parity of the W8A8 per-tensor static INT8 linear: bit-exact against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, to_dev_bf16, to_dev, bf16_bits, workspace

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("tile", [0, 1, 3, 4, 6, 8, 11, 13, 14])
@pytest.mark.parametrize("shape", [(1, 4096, 264), (16, 1024, 512), (64, 2048, 136), (200, 512, 392),
                                   (512, 768, 256), (33, 11008, 72), (17, 1024, 200), (32, 640, 136),
                                   (48, 4096, 520), (64, 11008, 264), (5, 192, 8)])
def test_w8a8_bit_exact(shape, tile):
    M, K, N = shape
    say("w8a8 M=%d K=%d N=%d tile=%d" % (M, K, N, tile))
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    # activations are quantized on the GPU, weights offline (here: by the oracle)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    tw.tweo_quantize_i8(to_dev_bf16(x), inv_x, xq)
    oxq = oracle.quantize_i8(x, inv_x)
    assert np.array_equal(xq.cpu().numpy(), oxq)
    owq = oracle.quantize_i8(w, inv_w)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_set_gemm_tile(tile)
    try:
        tw.tweo_w8a8_linear(xq, to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    assert np.array_equal(bf16_bits(y), want)


@pytest.mark.parametrize("shape", [(512, 1024, 768), (1024, 512, 512), (4352, 1024, 4096)])
def test_w8a8_deferred_epilogue_kernel_bit_exact(shape):
    # whole 256x256 tiles: the shapes the deferred-epilogue kernel (variant 15) takes; the last
    # one gives some workgroups two tiles on a 256-CU machine
    M, K, N = shape
    say("w8a8 deferred M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_set_gemm_tile(15)
    try:
        tw.tweo_w8a8_linear(to_dev(oxq), to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    assert np.array_equal(bf16_bits(y), oracle.w8a8_linear(oxq, owq, alpha))


@pytest.mark.parametrize("shape", [(4, 4096, 8192), (16, 1024, 8200), (17, 2048, 8192), (33, 4096, 12288),
                                   (64, 64, 8192), (48, 640, 16384), (64, 4096, 8192), (5, 192, 8200)])
def test_w8a8_weight_streaming_kernel_wide_outputs_bit_exact(shape):
    # M <= 64 with many blocks of weight rows per workgroup (two to four, and a second pass); ragged M
    # and N, K shorter than a stage and K that ends inside one
    M, K, N = shape
    say("w8a8 weight streaming, wide M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_w8a8_linear(to_dev(oxq), to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits(y), oracle.w8a8_linear(oxq, owq, alpha))


@pytest.mark.parametrize("shape", [(1, 1024, 24), (5, 1088, 48), (16, 4160, 4104), (17, 1024, 200), (33, 11008, 72),
                                   (64, 11008, 4104), (64, 2048, 16384), (8, 1024, 20480), (40, 3072, 12288),
                                   (64, 1024, 8), (32, 5120, 5000), (64, 64, 8192), (3, 192, 40), (48, 320, 264)])
def test_w8a8_weight_streaming_kernel_forced_bit_exact(shape):
    # the weight-streaming kernel (forced: variant 17): every M block count, 1 to 4 weight blocks per
    # workgroup and a second pass (20480 rows), K that ends inside a stage (1088, 4160, 11008,
    # 5120), ragged M and N; twice, the second call finding the first one's LDS and outputs
    M, K, N = shape
    say("w8a8 weight streaming, forced M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    for rep in range(2):
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
        tw.tweo_set_gemm_tile(17)
        try:
            tw.tweo_w8a8_linear(to_dev(oxq), to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
            torch.cuda.synchronize()
        finally:
            tw.tweo_set_gemm_tile(0)
        assert np.array_equal(bf16_bits(y), want)


def test_w8a8_stream_k_bit_exact():
    # 64 tiles, long K, K-split switched on: int32 partial accumulators are added exactly, so the
    # result is the same bits as the plain schedule's and the oracle's
    M, K, N = 2048, 8192, 2048
    say("w8a8 stream-K M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    for on in (True, False):
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
        tw.tweo_set_stream_k(on)
        try:
            tw.tweo_w8a8_linear(to_dev(oxq), to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
            torch.cuda.synchronize()
        finally:
            tw.tweo_set_stream_k(False)
        assert np.array_equal(bf16_bits(y), want)


def test_w8a8_extreme_accumulators():
    # +-127 everywhere: |acc| = 127*127*K exceeds 2^24, exercising the int32 -> fp32 rounding
    M, K, N = 64, 11008, 128
    say("w8a8 extreme M=%d K=%d N=%d" % (M, K, N))
    xq = np.full((M, K), 127, np.int8)
    wq = np.full((N, K), -127, np.int8)
    wq[::2] = 127
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_w8a8_linear(to_dev(xq), to_dev(wq), 1.0, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
    assert np.array_equal(bf16_bits(y), oracle.w8a8_linear(xq, wq, 1.0))


@pytest.mark.parametrize("tile", [0, 17])
@pytest.mark.parametrize("shape", [(65, 1024, 72), (96, 2048, 136), (100, 11008, 264), (128, 4096, 520),
                                   (128, 640, 4104), (80, 192, 8), (128, 4096, 12288), (128, 11008, 4096),
                                   (112, 4096, 11008)])
def test_w8a8_weight_streaming_up_to_128_rows(shape, tile):
    # 64 < M <= 128 on the weight-streaming kernel (eight blocks of 16 rows of X): one to four blocks
    # of weight rows per workgroup, ragged M, N and K (K a multiple of 64 only), the 7B shapes
    M, K, N = shape
    say("w8a8 streaming M=%d K=%d N=%d tile=%d" % (M, K, N, tile))
    x, w = synth.w8a8_inputs(1, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_set_gemm_tile(tile)
    try:
        tw.tweo_w8a8_linear(to_dev(oxq), to_dev(owq), alpha, y, workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K))
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    assert np.array_equal(bf16_bits(y), want)
    if tile == 0:
        # per-token and per-channel steps take the same kernel
        sx = torch.full((M,), float(ax / np.float32(127.0)), dtype=torch.float32, device=DEV)
        sw = torch.full((N,), float(aw / np.float32(127.0)), dtype=torch.float32, device=DEV)
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)
        tw.tweo_w8a8_linear_scaled(to_dev(oxq), to_dev(owq), sx, sw, y)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits(y), oracle.w8a8_linear_scaled(oxq, owq, sx.cpu().numpy(), sw.cpu().numpy()))


@pytest.mark.parametrize("shape", [(256, 11008, 4096), (512, 8192, 256), (256, 16384, 512), (512, 11008, 4096),
                                   (1024, 10240, 2816)])
def test_w8a8_k_split_of_whole_tiles(shape):
    # few whole 256x256 tiles under a contraction of 8192 and more: workgroups share a tile's K, the
    # int32 runs are added exactly by a second kernel (with the workspace tweo_workspace_bytes asks
    # for); without a workspace the tiled kernels run - both must give the oracle's bits
    M, K, N = shape
    say("w8a8 k-split tiles M=%d K=%d N=%d" % (M, K, N))
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_W8A8_LINEAR, M, N, K) >= 2 * M * N * 4
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    xd, wd = to_dev(oxq), to_dev(owq)
    ws = torch.full((tw.tweo_workspace_bytes(tw.TWEO_OP_W8A8_LINEAR, M, N, K),), 0xEE, dtype=torch.uint8, device=DEV)
    for w_arg in (ws, ws, None):
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
        tw.tweo_w8a8_linear(xd, wd, alpha, y, w_arg)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits(y), want)


@pytest.mark.parametrize("shape", [(192, 11008, 4096), (256, 8192, 2048), (160, 8192, 520), (200, 16384, 264),
                                   (129, 8192, 8), (256, 11008, 4096)])
def test_w8a8_weight_streaming_up_to_256_rows_into_a_narrow_projection(shape):
    # 128 < M <= 256, K >= 8192, at most one block of 16 weight rows per CU: twelve or sixteen blocks
    # of rows of X beside the weight rows.  With a workspace, M = 256 on whole tiles takes the K split
    # of the tiled kernel instead; without one the weight-streaming kernel: the same bits either way.
    M, K, N = shape
    say("w8a8 streaming (narrow) M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(2, M, K=K, N=N)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    inv_x, inv_w = np.float32(127.0) / ax, np.float32(127.0) / aw
    alpha = (ax / np.float32(127.0)) * (aw / np.float32(127.0))
    oxq, owq = oracle.quantize_i8(x, inv_x), oracle.quantize_i8(w, inv_w)
    want = oracle.w8a8_linear(oxq, owq, alpha)
    xd, wd = to_dev(oxq), to_dev(owq)
    for w_arg in (workspace(tw.TWEO_OP_W8A8_LINEAR, M, N, K), None):
        y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
        tw.tweo_w8a8_linear(xd, wd, alpha, y, w_arg)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits(y), want)
    # per-token and per-channel steps take the same kernel
    sx = torch.full((M,), float(ax / np.float32(127.0)), dtype=torch.float32, device=DEV)
    sw = torch.full((N,), float(aw / np.float32(127.0)), dtype=torch.float32, device=DEV)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)
    tw.tweo_w8a8_linear_scaled(xd, wd, sx, sw, y)
    torch.cuda.synchronize()
    want_v = oracle.w8a8_linear_scaled(oxq, owq, sx.cpu().numpy(), sw.cpu().numpy())
    assert np.array_equal(bf16_bits(y), want_v)
