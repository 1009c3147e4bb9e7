"""GPU parity, HBM-bound passes: amax, E4M3 quantize-cast (+transpose), INT8 quantize.
Bit-exact against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, to_dev_bf16, to_dev, scalar_f32, gpu_amax, gpu_quantize

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("n", [1, 7, 8, 9, 1000, 8191, 256 * 512, 3 * 1024 * 1024 + 5])
def test_amax_sizes(n):
    say("amax n=%d" % n)
    rng = np.random.default_rng(n)
    x = synth.f32_to_bf16_bits((rng.standard_normal(n) * 3).astype(np.float32))
    if n > 100:
        x[rng.integers(0, n)] = synth.f32_to_bf16_bits(np.array([-7777.0], np.float32))[0]
    # an offset view keeps the 16-byte alignment the ABI asks for
    got = gpu_amax(to_dev_bf16(x)).cpu().numpy()[0]
    assert got.view(np.uint32) == np.float32(oracle.amax_bf16(x)).view(np.uint32)


def test_amax_edge_values_and_overwrite():
    say("amax edges")
    for bits in ([0, 0x8000, 0], [0x3F80, 0xFF80, 0x4000], [0x3F80, 0x7F80, 0x7FC1], [0x0001, 0x8002]):
        x = np.array(bits * 8, np.uint16)
        got = gpu_amax(to_dev_bf16(x)).cpu().numpy()[0]
        want = np.float32(oracle.amax_bf16(x))
        assert got.view(np.uint32) == want.view(np.uint32), bits
    # result does not depend on what the output held before (it is overwritten, not max-ed)
    x = synth.f32_to_bf16_bits(np.full(64, 0.5, np.float32))
    out = scalar_f32(1e9)
    tw.tweo_amax(to_dev_bf16(x), out)
    assert out.cpu().numpy()[0] == 0.5


def test_quantize_all_bf16_patterns_times_scales():
    # every bf16 bit pattern, for scales that exercise flush, subnormal, normal, saturate
    allx = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(256, 256)
    amaxes = [448.0, 1.0, 9873.0, 3.0e4, 0.013, 1e-30, 3.0e38, 448.0 * 8, 5000.0, 0.0, np.inf, np.nan]
    xd = to_dev_bf16(allx)
    for amax in amaxes:
        say("quantize all patterns, amax=%r" % amax)
        a = scalar_f32(amax)
        q, qT, s, si = gpu_quantize(xd, a)
        scale, scale_inv = oracle.scale_from_amax(np.float32(amax))
        assert s.cpu().numpy()[0] == scale and si.cpu().numpy()[0] == scale_inv
        want, wantT = oracle.quantize_e4m3(allx, scale)
        got, gotT = q.cpu().numpy(), qT.cpu().numpy()
        nan = (want & 0x7F) == 0x7F
        assert np.array_equal((got & 0x7F) == 0x7F, nan)  # NaN -> NaN code (sign unpinned)
        assert np.array_equal(got[~nan], want[~nan])
        assert np.array_equal(gotT, got.T)


@pytest.mark.parametrize("shape", [(256, 512), (512, 512), (1, 8), (3, 16), (61, 72), (200, 264),
                                   (129, 1024), (64, 256), (8, 2048)])
def test_quantize_shapes_ragged(shape):
    say("quantize shape", shape)
    r, c = shape
    x, _, _ = synth.fp8_linear_inputs(0, 0, M=r, K=c, N=8)
    xd = to_dev_bf16(x)
    a = gpu_amax(xd)
    amax = oracle.amax_bf16(x)
    assert a.cpu().numpy()[0] == amax
    scale, _ = oracle.scale_from_amax(amax)
    want, wantT = oracle.quantize_e4m3(x, scale)
    q, qT, _, _ = gpu_quantize(xd, a)
    assert np.array_equal(q.cpu().numpy(), want)
    assert np.array_equal(qT.cpu().numpy(), wantT)
    q2, _, _, _ = gpu_quantize(xd, a, transpose=False)
    assert np.array_equal(q2.cpu().numpy(), want)


def test_quantize_outputs_untouched_outside():
    say("quantize guard bytes")
    r, c = 61, 72
    x, _, _ = synth.fp8_linear_inputs(0, 0, M=r, K=c, N=8)
    xd = to_dev_bf16(x)
    a = gpu_amax(xd)
    qbuf = torch.full((r * c + 64,), 0xAB, dtype=torch.uint8, device=DEV)
    tbuf = torch.full((r * c + 64,), 0xCD, dtype=torch.uint8, device=DEV)
    tw.tweo_quantize_e4m3(xd, a, qbuf[: r * c].view(r, c), tbuf[: r * c].view(c, r))
    assert (qbuf[r * c:] == 0xAB).all() and (tbuf[r * c:] == 0xCD).all()


@pytest.mark.parametrize("n", [8, 64, 4096, 16 * 4096, 64 * 11008, 1000 * 8])
def test_quantize_i8(n):
    say("quantize_i8 n=%d" % n)
    x, _ = synth.w8a8_inputs(0, 1, K=n, N=8)
    x = x.reshape(-1)
    x[:6] = synth.f32_to_bf16_bits(np.array([0.5, 1.5, 2.5, -0.5, 300.0, -300.0], np.float32))[: min(6, n)]
    for inv_step in (np.float32(127.0) / oracle.amax_bf16(x), np.float32(1.0), np.float32(40.0)):
        out = torch.empty(n, dtype=torch.int8, device=DEV)
        tw.tweo_quantize_i8(to_dev_bf16(x), inv_step, out)
        assert np.array_equal(out.cpu().numpy(), oracle.quantize_i8(x, inv_step))
    special = np.array([0x7FC0, 0x7F80, 0xFF80, 0x0000, 0x8000, 0x3F00, 0xBF00, 0x4300], np.uint16)
    out = torch.empty(8, dtype=torch.int8, device=DEV)
    tw.tweo_quantize_i8(to_dev_bf16(special), 1.0, out)
    assert np.array_equal(out.cpu().numpy(), oracle.quantize_i8(special, 1.0))
