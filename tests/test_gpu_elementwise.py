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


@pytest.mark.parametrize("pen,g", [((3.0, 1e-6, 4), 1e-3), ((3.0, 1e-6, 4), 0.5), ((2.0, 0.0, 2), 0.1),
                                   ((4.0, 1e-6, 3), 0.05), ((3.0, 1e-6, 1), 0.2)])
def test_penalty_gradient_injection(pen, g):
    # dy' = dy + d(penalty)/da (the derivative of the loss of Sec. 3.3), fp32 on the GPU against
    # the fp64 oracle: within bf16 output rounding plus the fp32 arithmetic in front of it
    n = 256 * 1024 + 8
    say("penalty gradient injection", pen, g)
    rng = np.random.default_rng(int(pen[2]) * 7 + 1)
    a = synth.f32_to_bf16_bits((rng.standard_normal(n) * 6).astype(np.float32))
    a[:6] = [0x0000, 0x8000, 0x4110, 0xC110, 0x4680, 0xC680]  # +-0, +-9, +-16384
    dy = synth.f32_to_bf16_bits(rng.standard_normal(n).astype(np.float32))
    want_bits, exact = oracle.penalty_grad_inject(dy, a, *pen, g=g)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    tw.tweo_penalty_grad_inject(to_dev_bf16(dy), to_dev_bf16(a), pen, g, out)
    torch.cuda.synchronize()
    got_bits = out.view(torch.int16).cpu().numpy().view(np.uint16)
    got = synth.bf16_bits_to_f32(got_bits).astype(np.float64)
    d = synth.bf16_bits_to_f32(dy).astype(np.float64)
    # 2^-9 relative for the rounding to bf16, 2^-20 of each term for the fp32 arithmetic
    tol = 2.0 ** -8 * np.abs(exact) + 2.0 ** -20 * (np.abs(d) + np.abs(exact - d)) + 1e-30
    assert np.all(np.abs(got - exact) <= tol)
    assert np.mean(got_bits == want_bits) > 0.99  # all but the odd boundary case are the same bits
    assert got[0] == d[0] and got[1] == d[1]       # sign(0) = 0
    # in place
    buf = to_dev_bf16(dy).clone()
    tw.tweo_penalty_grad_inject(buf, to_dev_bf16(a), pen, g, buf)
    torch.cuda.synchronize()
    assert np.array_equal(buf.view(torch.int16).cpu().numpy().view(np.uint16), got_bits)


@pytest.mark.parametrize("shape", [(256, 512), (200, 136), (48, 4096), (1024, 768)])
def test_delayed_scaling_sequence(shape):
    # 20 steps of the delayed-scaling cast (Sec. 4.3: amax history of length 16) with a spike at
    # step 3: bytes, transposed bytes and every word of the state bit-exact against the oracle
    rows, cols = shape
    say("delayed scaling", shape)
    ref = oracle.DelayedScaling()
    state = torch.full((tw.DELAYED_STATE_WORDS,), -7.0, dtype=torch.float32, device=DEV)
    tw.tweo_delayed_state_init(state)
    q = torch.empty((rows, cols), dtype=torch.uint8, device=DEV)
    qT = torch.empty((cols, rows), dtype=torch.uint8, device=DEV)
    rng = np.random.default_rng(rows + cols)
    for step in range(20):
        v = (rng.standard_normal((rows, cols)) * (1.0 + 0.1 * step)).astype(np.float32)
        if step == 3:
            v[rng.integers(rows), rng.integers(cols)] = -4321.0
        if step == 7:
            v[:] = 0.0      # an all-zero tensor: amax 0 enters the history
        x = synth.f32_to_bf16_bits(v)
        oq, oqT, used, used_inv = ref.cast(x)
        q.fill_(0x55)
        qT.fill_(0x55)
        tw.tweo_quantize_e4m3_delayed(to_dev_bf16(x), state, q, qT, bootstrap=(step == 0))
        torch.cuda.synchronize()
        st = state.cpu().numpy()
        assert np.array_equal(q.cpu().numpy(), oq), step
        assert np.array_equal(qT.cpu().numpy(), oqT), step
        assert st[tw.DELAYED_USED_SCALE].view(np.uint32) == np.float32(used).view(np.uint32), step
        assert st[tw.DELAYED_USED_SCALE_INV].view(np.uint32) == np.float32(used_inv).view(np.uint32), step
        assert st[tw.DELAYED_NEXT_SCALE].view(np.uint32) == np.float32(ref.next_scale).view(np.uint32), step
        assert st[16] == 0.0                                   # accumulator cleared
        assert int(st[20:21].view(np.uint32)[0]) == len(ref.history)
        ring = np.sort(st[:16].view(np.uint32))[::-1][:len(ref.history)]
        want = np.sort(np.array(ref.history, np.float32).view(np.uint32))[::-1]
        assert np.array_equal(ring, want), step


def test_delayed_scaling_state_checkpoint_and_restore():
    # The 32-word state is the only state of the recipe (Sec. 4.3: amax history of length 16).
    # Copy it to the host in the middle of a 20-step sequence, restore it into a fresh buffer and
    # continue there: bytes and every state word equal the uninterrupted run and the oracle.
    rows, cols = 256, 512
    ref = oracle.DelayedScaling()
    state = torch.full((tw.DELAYED_STATE_WORDS,), -7.0, dtype=torch.float32, device=DEV)
    tw.tweo_delayed_state_init(state)
    resumed = None
    rng = np.random.default_rng(99)
    q = torch.empty((rows, cols), dtype=torch.uint8, device=DEV)
    qT = torch.empty((cols, rows), dtype=torch.uint8, device=DEV)
    q2, qT2 = torch.empty_like(q), torch.empty_like(qT)
    for step in range(20):
        v = (rng.standard_normal((rows, cols)) * (1.0 + 0.3 * step)).astype(np.float32)
        if step in (5, 12):
            v[rng.integers(rows), rng.integers(cols)] = 2500.0 * (step - 4)
        x = synth.f32_to_bf16_bits(v)
        oq, oqT, used, used_inv = ref.cast(x)
        tw.tweo_quantize_e4m3_delayed(to_dev_bf16(x), state, q, qT, bootstrap=(step == 0))
        if resumed is not None:
            tw.tweo_quantize_e4m3_delayed(to_dev_bf16(x), resumed, q2, qT2, bootstrap=False)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), oq) and np.array_equal(qT.cpu().numpy(), oqT), step
        if resumed is not None:
            assert torch.equal(q, q2) and torch.equal(qT, qT2), step
            assert torch.equal(state.view(torch.int32), resumed.view(torch.int32)), step
        if step == 9:
            saved = state.cpu().numpy().copy()                  # the checkpoint: 128 bytes
            assert saved.nbytes == tw.tweo_delayed_state_bytes()
            resumed = torch.from_numpy(saved).to(DEV)           # a fresh buffer
        st = state.cpu().numpy()
        assert st[tw.DELAYED_USED_SCALE].view(np.uint32) == np.float32(used).view(np.uint32), step
        assert st[tw.DELAYED_NEXT_SCALE].view(np.uint32) == np.float32(ref.next_scale).view(np.uint32), step
        assert not st[23:].view(np.uint32).any()                # words beyond the documented ones stay 0
