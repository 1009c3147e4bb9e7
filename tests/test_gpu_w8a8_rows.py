"""GPU parity of the finer INT8 granularities (Sec. 4.4: per-token activations, per-channel weights):
row-granular AbsMax quantisation and the W8A8 linear with step vectors, bit-exact against the CPU
oracle through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, to_dev_bf16, to_dev, bf16_bits

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def gpu_quantize_rows(x_bits, eps):
    rows, cols = x_bits.shape
    q = torch.full((rows, cols), 99, dtype=torch.int8, device=DEV)
    step = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    tw.tweo_quantize_i8_rows(to_dev_bf16(x_bits), eps, q, step)
    torch.cuda.synchronize()
    return q.cpu().numpy(), step.cpu().numpy()


def same_steps(a, b):
    return np.array_equal(a.view(np.uint32)[~np.isnan(a)], b.view(np.uint32)[~np.isnan(b)]) and \
        np.array_equal(np.isnan(a), np.isnan(b))


# one wave per row (cols <= 2048: all in registers; ragged row counts), a workgroup per row (all
# in registers up to 8192, a second read beyond), the 7B shapes' row lengths
@pytest.mark.parametrize("shape", [(1, 8), (3, 24), (5, 520), (64, 2048), (67, 2040), (16, 2056), (9, 4096),
                                   (4, 8192), (3, 8200), (2, 11008), (2, 65536), (4096, 512), (1031, 4096)])
@pytest.mark.parametrize("eps", [0.0, 1e-6])
def test_quantize_rows(shape, eps):
    rows, cols = shape
    say("quantize_i8_rows %dx%d eps=%g" % (rows, cols, eps))
    rng = np.random.default_rng(rows * 7919 + cols)
    x = rng.standard_normal((rows, cols)) * np.exp(rng.uniform(-6, 6, (rows, 1)))
    x[rng.random((rows, cols)) < 0.001] *= 50.0  # a few outliers that set their row's step
    xb = synth.f32_to_bf16_bits(x.astype(np.float32))
    q, step = gpu_quantize_rows(xb, eps)
    oq, ostep = oracle.quantize_i8_rows(xb, eps)
    assert np.array_equal(step.view(np.uint32), ostep.view(np.uint32))
    assert np.array_equal(q, oq)


def test_quantize_rows_all_bf16_patterns_and_special_rows():
    # every bf16 pattern as an element, for rows whose maximum is set by one planted value
    allx = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = allx[(allx & 0x7F80) != 0x7F80]
    rows = []
    for top in (1.0, 3.0e-3, 777.0, 3.0e38, 1e-38, 2.5e-40):
        body = finite[(finite & 0x7FFF) <= synth.f32_to_bf16_bits(np.array([top], np.float32))[0]]
        pad = (-body.size) % 8
        rows.append(np.concatenate([body, np.zeros(pad, np.uint16)]))
    for r in rows:
        say("all patterns up to a planted maximum, %d elements" % r.size)
        for eps in (0.0, 1e-6):
            q, step = gpu_quantize_rows(r[None, :], eps)
            oq, ostep = oracle.quantize_i8_rows(r[None, :], eps)
            assert same_steps(step, ostep) and np.array_equal(q, oq)
    # zero row, NaN row, Inf row, ordinary row in one matrix: each row on its own
    t = synth.f32_to_bf16_bits(np.array([[0] * 8, [1, -2, 0.5, np.nan, 0, 0, 0, 0],
                                         [3, -np.inf, 1, 0, 0, 0, 0, 0], [1, -4, 0.5, 2, 0, 0, 0, 3]], np.float32))
    for eps in (0.0, 0.5):
        q, step = gpu_quantize_rows(t, eps)
        oq, ostep = oracle.quantize_i8_rows(t, eps)
        assert same_steps(step, ostep) and np.array_equal(q, oq)


def run_scaled(xq, wq, sx, sw, tile=0):
    M, N = xq.shape[0], wq.shape[0]
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)  # poisoned
    tw.tweo_set_gemm_tile(tile)
    try:
        tw.tweo_w8a8_linear_scaled(to_dev(xq), to_dev(wq), to_dev(np.atleast_1d(sx).astype(np.float32)),
                                   to_dev(np.atleast_1d(sw).astype(np.float32)), y)
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    return bf16_bits(y)


GRAN = ["KC", "KT", "TC", "TT"]  # activations per token (K) / tensor (T) x weights per channel (C) / tensor (T)


def quantised(M, K, N, gran):
    x, w = synth.w8a8_inputs(0, M, K=K, N=N)
    if gran[0] == "K":
        xq, sx = oracle.quantize_i8_rows(x, 1e-6)
    else:
        ax = oracle.amax_bf16(x)
        xq, sx = oracle.quantize_i8(x, np.float32(127.0) / ax), np.array([ax / np.float32(127.0)], np.float32)
    if gran[1] == "C":
        wq, sw = oracle.quantize_i8_rows(w, 1e-6)
    else:
        aw = oracle.amax_bf16(w)
        wq, sw = oracle.quantize_i8(w, np.float32(127.0) / aw), np.array([aw / np.float32(127.0)], np.float32)
    return xq, wq, sx, sw


# the weight-streaming kernel (M <= 64, every M block / N block variant, ragged N), then the tiled
# kernels on ragged and whole-tile shapes
@pytest.mark.parametrize("gran", GRAN)
@pytest.mark.parametrize("shape", [(1, 4096, 264), (16, 1024, 512), (17, 1024, 200), (32, 640, 136),
                                   (48, 4096, 520), (64, 2048, 136), (64, 4096, 8192), (8, 4096, 8192), (20, 640, 8200),
                                   (200, 512, 392), (512, 768, 256), (1024, 1024, 1024)])
def test_scaled_linear_bit_exact(shape, gran):
    M, K, N = shape
    say("w8a8 scaled M=%d K=%d N=%d %s" % (M, K, N, gran))
    xq, wq, sx, sw = quantised(M, K, N, gran)
    got = run_scaled(xq, wq, sx, sw)
    assert np.array_equal(got, oracle.w8a8_linear_scaled(xq, wq, sx, sw))


@pytest.mark.parametrize("gran", ["KC", "TT"])
@pytest.mark.parametrize("shape", [(5, 1088, 48), (33, 11008, 72), (64, 2048, 16384), (16, 4160, 4104)])
def test_scaled_linear_weight_streaming_kernel_forced(shape, gran):
    # the same with the weight-streaming kernel forced (variant 17), bf16 and INT8 outputs
    M, K, N = shape
    say("w8a8 scaled, weight streaming forced M=%d K=%d N=%d %s" % (M, K, N, gran))
    xq, wq, sx, sw = quantised(M, K, N, gran)
    assert np.array_equal(run_scaled(xq, wq, sx, sw, tile=17), oracle.w8a8_linear_scaled(xq, wq, sx, sw))
    inv_out = np.float32(127.0) / np.float32(1.5)
    yq = torch.full((M, N), 99, dtype=torch.int8, device=DEV)
    tw.tweo_set_gemm_tile(17)
    try:
        tw.tweo_w8a8_linear_scaled_i8out(to_dev(xq), to_dev(wq), to_dev(np.atleast_1d(sx).astype(np.float32)),
                                         to_dev(np.atleast_1d(sw).astype(np.float32)), inv_out, yq)
        torch.cuda.synchronize()
    finally:
        tw.tweo_set_gemm_tile(0)
    assert np.array_equal(yq.cpu().numpy(), oracle.w8a8_linear_scaled_i8out(xq, wq, sx, sw, inv_out))


@pytest.mark.parametrize("tile", [1, 3, 4, 6, 8, 11, 13, 14, 15, 16])
@pytest.mark.parametrize("shape", [(200, 512, 392), (768, 2048, 512)])
def test_scaled_linear_every_tiled_kernel(shape, tile):
    # forced variants; 15 and 16 (per-tensor only kernels) must fall back, not ignore the vectors
    M, K, N = shape
    say("w8a8 scaled M=%d K=%d N=%d tile=%d" % (M, K, N, tile))
    xq, wq, sx, sw = quantised(M, K, N, "KC")
    got = run_scaled(xq, wq, sx, sw, tile)
    assert np.array_equal(got, oracle.w8a8_linear_scaled(xq, wq, sx, sw))


def test_quantise_and_multiply_on_the_gpu_end_to_end():
    # W8(C)A8(K) as a serving step would run it: weights per channel offline, tokens on the fly
    M, K, N = 48, 4096, 1024
    say("w8a8 W(C)A(K) end to end M=%d K=%d N=%d" % (M, K, N))
    x, w = synth.w8a8_inputs(1, M, K=K, N=N)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    wq = torch.empty((N, K), dtype=torch.int8, device=DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=DEV)
    sw = torch.empty((N,), dtype=torch.float32, device=DEV)
    y = torch.full((M, N), float('nan'), dtype=torch.bfloat16, device=DEV)
    tw.tweo_quantize_i8_rows(to_dev_bf16(w), 1e-6, wq, sw)
    tw.tweo_quantize_i8_rows(to_dev_bf16(x), 1e-6, xq, sx)
    tw.tweo_w8a8_linear_scaled(xq, wq, sx, sw, y)
    torch.cuda.synchronize()
    oxq, osx = oracle.quantize_i8_rows(x, 1e-6)
    owq, osw = oracle.quantize_i8_rows(w, 1e-6)
    assert np.array_equal(bf16_bits(y), oracle.w8a8_linear_scaled(oxq, owq, osx, osw))


def test_error_paths():
    x = torch.zeros((8, 16), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((8, 16), dtype=torch.int8, device=DEV)
    st = torch.zeros((8,), dtype=torch.float32, device=DEV)
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_quantize_i8_rows(x, -1.0, q, st)
    assert e.value.status == tw.TWEO_ERR_INVALID_ARG
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_quantize_i8_rows(x[:, :12].contiguous(), 0.0, q, st)
    assert e.value.status == tw.TWEO_ERR_UNSUPPORTED
    y = torch.zeros((8, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(ValueError):
        tw.tweo_w8a8_linear_scaled(q, q, st[:3], st, y)


# INT8 output for a quantised residual stream: the weight-streaming kernel (one and several
# weight blocks per workgroup), the tiled kernels on ragged and whole-tile shapes; steps that leave most values in
# range, and one that saturates
@pytest.mark.parametrize("gran", ["KC", "TT"])
@pytest.mark.parametrize("shape", [(1, 4096, 264), (17, 1024, 200), (64, 2048, 136), (64, 4096, 8192), (8, 4096, 8192),
                                   (200, 512, 392), (1024, 1024, 1024)])
def test_scaled_linear_int8_output_bit_exact(shape, gran):
    M, K, N = shape
    say("w8a8 int8 out M=%d K=%d N=%d %s" % (M, K, N, gran))
    xq, wq, sx, sw = quantised(M, K, N, gran)
    ref = synth.bf16_bits_to_f32(oracle.w8a8_linear_scaled(xq, wq, sx, sw))
    s_out = np.float32(np.abs(ref).max())
    for inv in (np.float32(127.0) / s_out, np.float32(127.0) / (s_out / np.float32(16.0))):
        yq = torch.full((M, N), 99, dtype=torch.int8, device=DEV)  # poisoned
        tw.tweo_w8a8_linear_scaled_i8out(to_dev(xq), to_dev(wq), to_dev(np.atleast_1d(sx).astype(np.float32)),
                                         to_dev(np.atleast_1d(sw).astype(np.float32)), inv, yq)
        torch.cuda.synchronize()
        want = oracle.w8a8_linear_scaled_i8out(xq, wq, sx, sw, inv)
        assert np.array_equal(yq.cpu().numpy(), want)
        assert np.abs(want).max() == 127
