"""GPU parity of the whole FP8 linear under the paper's own recipe (Sec. 4.3: per-tensor delayed
scaling with an amax history of 16, E4M3 forward tensors, E4M3 or E5M2 gradients) through the two
bf16 entry points, over a sequence of steps on one set of states."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_23225_amd as tw
from paper_2511_23225_amd import synth
from gpu_util import DEV, PEN, to_dev_bf16, bf16_bits, workspace, check_gemm, check_penalty

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dy_e5m2", [False, True])
@pytest.mark.parametrize("shape", [(256, 512, 512), (1024, 1024, 768), (208, 256, 144)])
def test_delayed_scaling_linear_sequence(shape, dy_e5m2):
    M, K, N = shape
    ref_x, ref_w, ref_dy = oracle.DelayedScaling(), oracle.DelayedScaling(), oracle.DelayedScaling(e5m2=dy_e5m2)
    states = [torch.zeros(tw.DELAYED_STATE_WORDS, dtype=torch.float32, device=DEV) for _ in range(3)]
    for st in states:
        tw.tweo_delayed_state_init(st)
    u8 = lambda *s: torch.full(s, 0x55, dtype=torch.uint8, device=DEV)
    xq, xqT, wq, wqT, dyq, dyqT = u8(M, K), u8(K, M), u8(N, K), u8(K, N), u8(M, N), u8(N, M)
    sc = torch.full((16,), -3.0, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(xq, xqT, wq, wqT, sc)
    ws = workspace(tw.TWEO_OP_FP8_LINEAR_FWD, M, N, K)
    wsb = workspace(tw.TWEO_OP_FP8_LINEAR_BWD, M, N, K)
    rng = np.random.default_rng(M + N)
    x0, w0, dy0 = synth.fp8_linear_inputs(1, 0, M=M, K=K, N=N)
    for step in range(5):
        print("delayed linear", shape, "e5m2" if dy_e5m2 else "e4m3", "step", step, flush=True)
        # every step new activations and gradients (growing, with a spike at step 2), drifting weights
        gain = np.float32(1.0 + 0.5 * step)
        x = synth.f32_to_bf16_bits(np.roll(synth.bf16_bits_to_f32(x0), step, axis=0) * gain)
        dy = synth.f32_to_bf16_bits(np.roll(synth.bf16_bits_to_f32(dy0), step, axis=1) / gain)
        w = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(w0) * np.float32(1.0 + 0.01 * step))
        if step == 2:
            dy[rng.integers(M), rng.integers(N)] = synth.f32_to_bf16_bits(np.float32(300.0).reshape(1))[0]
        oxq, oxqT, sx, sxi = ref_x.cast(x)
        owq, owqT, sw, swi = ref_w.cast(w)
        odyq, odyqT, sdy, sdyi = ref_dy.cast(dy)
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        dx = torch.full((M, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        dw = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        S = torch.zeros(2, dtype=torch.float64, device=DEV)
        boot = step == 0
        tw.tweo_fp8_linear_fwd_bf16_delayed(to_dev_bf16(x), to_dev_bf16(w), y, saved, states[0], states[1],
                                            bootstrap=boot, pen=PEN, penalty_sum=S, workspace=ws)
        tw.tweo_fp8_linear_bwd_bf16_delayed(to_dev_bf16(dy), saved, states[2], K, dyq, dyqT, dx, dw, wsb,
                                            bootstrap=boot, dy_e5m2=dy_e5m2)
        torch.cuda.synchronize()
        for g, o in ((xq, oxq), (xqT, oxqT), (wq, owq), (wqT, owqT), (dyq, odyq), (dyqT, odyqT)):
            assert np.array_equal(g.cpu().numpy(), o), step
        want = np.array([oracle.amax_bf16(x), sx, sxi, oracle.amax_bf16(w), sw, swi, oracle.amax_bf16(dy), sdy, sdyi],
                        np.float32)
        assert np.array_equal(sc.cpu().numpy()[:9].view(np.uint32), want.view(np.uint32)), step
        for st, ref in zip(states, (ref_x, ref_w, ref_dy)):
            h = st.cpu().numpy()
            assert h[tw.DELAYED_NEXT_SCALE].view(np.uint32) == np.float32(ref.next_scale).view(np.uint32)
            assert h[16] == 0.0 and int(h[20:21].view(np.uint32)[0]) == len(ref.history)
        ref, refabs, refbf = oracle.fp8_linear_fwd(oxq, owq, sxi, swi)
        check_gemm(bf16_bits(y), ref, refabs, K, "fwd")
        check_penalty(float(S.cpu()[0]), bf16_bits(y), refbf, oracle.penalty_sum(refbf, *PEN), PEN, strict=False)
        dx_ref, dx_abs = oracle.fp8_linear_dgrad(odyq, owq, sdyi, swi, dy_e5m2=dy_e5m2)
        dw_ref, dw_abs = oracle.fp8_linear_wgrad(odyq, oxq, sdyi, sxi, dy_e5m2=dy_e5m2)
        check_gemm(bf16_bits(dx), dx_ref, dx_abs, N, "dgrad")
        check_gemm(bf16_bits(dw), dw_ref, dw_abs, M, "wgrad")


def test_delayed_linear_error_paths():
    t = torch.zeros((16, 16), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((16, 16), dtype=torch.uint8, device=DEV)
    sc = torch.zeros(16, dtype=torch.float32, device=DEV)
    st = torch.zeros(tw.DELAYED_STATE_WORDS, dtype=torch.float32, device=DEV)
    saved = tw.make_saved(q, q, q, q, sc)
    with pytest.raises(tw.TweoError) as e:   # the two tensors need states of their own
        tw.tweo_fp8_linear_fwd_bf16_delayed(t, t, t, saved, st, st)
    assert e.value.status == tw.TWEO_ERR_INVALID_ARG
    with pytest.raises(tw.TweoError) as e:
        tw.tweo_fp8_linear_bwd_bf16_delayed(t, saved, None, 16, q, q, t, t)
    assert e.value.status == tw.TWEO_ERR_INVALID_ARG
