"""Pins for the oracle's row-granular AbsMax INT8 functions (Sec. 4.4, Eq. 4 with per-token /
per-channel s): exact rationals, closed forms, invariances and a library integer matmul."""
from fractions import Fraction

import numpy as np

import oracle
from paper_2511_23225_amd import synth

F32 = np.float32


def bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def frac_round_half_even(fr):
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def test_rows_against_exact_rationals():
    # each step re-done with exact rationals around the fp32 roundings the definition names
    rng = np.random.default_rng(5)
    x = bf16(rng.standard_normal((6, 40)) * np.exp(rng.uniform(-3, 3, (6, 1))))
    for eps in (0.0, 1e-6, 0.25):
        q, step = oracle.quantize_i8_rows(x, eps)
        xf = synth.bf16_bits_to_f32(x)
        for r in range(x.shape[0]):
            s = F32(np.abs(xf[r]).max()) + F32(eps)           # fp32 add
            assert isinstance(s, np.floating)
            inv = F32(127.0) / s                               # fp32 division
            assert step[r] == s / F32(127.0)
            for c in range(x.shape[1]):
                prod = F32(xf[r, c]) * inv                     # fp32 multiply
                want = frac_round_half_even(Fraction(float(prod)))
                assert q[r, c] == max(-127, min(127, want)), (r, c)


def test_rows_end_points_and_half_step_bound():
    x, _ = synth.w8a8_inputs(0, 48, K=512, N=64)
    q, step = oracle.quantize_i8_rows(x, 0.0)
    xf = synth.bf16_bits_to_f32(x).astype(np.float64)
    for r in range(48):
        i = np.argmax(np.abs(xf[r]))
        assert abs(int(q[r, i])) == 127 and np.sign(q[r, i]) == np.sign(xf[r, i])  # Eq. 4: +-Q_8
        assert np.abs(q[r]).max() == 127
        # X_deq = X_q / Q_8 * s is within half a step of x (plus the fp32 roundings of inv and x*inv)
        err = np.abs(q[r].astype(np.float64) * float(step[r]) - xf[r])
        assert err.max() <= 0.5 * float(step[r]) * (1 + 1e-5)


def test_rows_are_independent_and_scale_free():
    rng = np.random.default_rng(9)
    base = rng.standard_normal((5, 64)).astype(np.float32)
    x = bf16(base)
    q0, s0 = oracle.quantize_i8_rows(x, 0.0)
    # a power of two on one row is exact in bf16: its codes stay, its step scales, others unmoved
    y = synth.bf16_bits_to_f32(x).copy()
    y[2] *= 64.0
    q1, s1 = oracle.quantize_i8_rows(bf16(y), 0.0)
    assert np.array_equal(q0, q1)
    assert s1[2] == s0[2] * 64 and np.array_equal(np.delete(s0, 2), np.delete(s1, 2))
    # each row alone gives what it gives inside the matrix; permuting rows permutes results
    for r in range(5):
        qr, sr = oracle.quantize_i8_rows(x[r:r + 1], 0.0)
        assert np.array_equal(qr[0], q0[r]) and sr[0] == s0[r]
    perm = np.array([3, 0, 4, 1, 2])
    qp, sp = oracle.quantize_i8_rows(x[perm], 0.0)
    assert np.array_equal(qp, q0[perm]) and np.array_equal(sp, s0[perm])


def test_single_row_is_the_per_tensor_quantiser():
    # granularity "one row" and granularity "whole tensor" coincide for a one-row tensor
    x, _ = synth.w8a8_inputs(1, 1, K=768, N=8)
    q, step = oracle.quantize_i8_rows(x, 0.0)
    amax = oracle.amax_bf16(x)
    assert np.array_equal(q, oracle.quantize_i8(x, F32(127.0) / amax))
    assert step[0] == amax / F32(127.0)


def test_rows_special_values():
    t = bf16([[0, 0, 0, 0], [1, -2, 0.5, np.nan], [3, -np.inf, 1, 0], [1e-30, -1e-30, 0, 5e-31]])
    q, step = oracle.quantize_i8_rows(t, 0.0)
    assert q[0].tolist() == [0, 0, 0, 0] and step[0] == 0.0
    assert q[1].tolist() == [0, 0, 0, 0] and np.isnan(step[1])          # a NaN poisons its row only
    assert q[2].tolist() == [0, 0, 0, 0] and np.isinf(step[2])          # inv = 0: x*0 = 0, inf*0 = NaN -> 0
    assert q[3].tolist() == [127, -127, 0, 64]
    # eps moves the end point below Q_8: s = 1 + 1 -> the maximum maps to round(127/2) = 64 (ties to even)
    q, step = oracle.quantize_i8_rows(bf16([[1.0, -0.5, 0.25, 0.0]]), 1.0)
    assert q[0].tolist() == [64, -32, 16, 0] and step[0] == F32(2.0) / F32(127.0)


def int_ref(xq, wq):
    return xq.astype(np.int64) @ wq.astype(np.int64).T


def test_scaled_linear_power_of_two_steps_is_exact():
    rng = np.random.default_rng(3)
    xq = rng.integers(-127, 128, (7, 96), dtype=np.int8)
    wq = rng.integers(-127, 128, (11, 96), dtype=np.int8)
    ex, ew = rng.integers(-12, 4, 7), rng.integers(-12, 4, 11)
    sx, sw = np.exp2(ex).astype(np.float32), np.exp2(ew).astype(np.float32)
    y = oracle.w8a8_linear_scaled(xq, wq, sx, sw)
    exact = int_ref(xq, wq).astype(np.float64) * np.exp2(ex)[:, None] * np.exp2(ew)[None, :]
    # |acc| < 2^24 and power-of-two steps: nothing rounds before the final bf16 rounding
    assert np.array_equal(y, bf16(exact.astype(np.float32)))
    # the transposed problem swaps the roles of the two step vectors
    yt = oracle.w8a8_linear_scaled(wq, xq, sw, sx)
    assert np.array_equal(yt, y.T)


def test_scaled_linear_general_steps_against_library():
    x, w = synth.w8a8_inputs(2, 24, K=640, N=40)
    xq, sx = oracle.quantize_i8_rows(x, 1e-6)
    wq, sw = oracle.quantize_i8_rows(w, 1e-6)
    y = synth.bf16_bits_to_f32(oracle.w8a8_linear_scaled(xq, wq, sx, sw)).astype(np.float64)
    exact = int_ref(xq, wq) * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    # two fp32 roundings (2^-24 each) and one bf16 rounding (half an ulp of 8 significant bits: 2^-8)
    assert np.all(np.abs(y - exact) <= np.abs(exact) * (2.0 ** -8 + 2.0 ** -22))
    # dequantised product approximates the real one: per-element quantisation noise of both operands
    real = synth.bf16_bits_to_f32(x).astype(np.float64) @ synth.bf16_bits_to_f32(w).astype(np.float64).T
    rel = np.linalg.norm(y - real) / np.linalg.norm(real)
    assert rel < 0.02


def test_scaled_linear_per_tensor_steps_reduce_to_the_static_path():
    x, w = synth.w8a8_inputs(0, 16, K=512, N=64)
    ax, aw = oracle.amax_bf16(x), oracle.amax_bf16(w)
    xq = oracle.quantize_i8(x, F32(127.0) / ax)
    wq = oracle.quantize_i8(w, F32(127.0) / aw)
    # powers of two make (acc*sx)*sw == acc*(sx*sw) exactly, so both entry points must agree bit for bit
    sx, sw = F32(2.0 ** -5), F32(2.0 ** -9)
    assert np.array_equal(oracle.w8a8_linear_scaled(xq, wq, [sx], [sw]), oracle.w8a8_linear(xq, wq, sx * sw))
    # a length-1 vector broadcasts: same as the constant vector
    sx, sw = ax / F32(127.0), aw / F32(127.0)
    assert np.array_equal(oracle.w8a8_linear_scaled(xq, wq, [sx], [sw]),
                          oracle.w8a8_linear_scaled(xq, wq, np.full(16, sx, F32), np.full(64, sw, F32)))


def test_i8out_power_of_two_steps_against_exact_rationals():
    rng = np.random.default_rng(8)
    xq = rng.integers(-127, 128, (5, 64), dtype=np.int8)
    wq = rng.integers(-127, 128, (9, 64), dtype=np.int8)
    ex, ew = rng.integers(-10, -6, 5), rng.integers(-9, -5, 9)
    sx, sw = np.exp2(ex).astype(np.float32), np.exp2(ew).astype(np.float32)
    inv = F32(127.0) / F32(3.0)                     # s_out = 3: a non-trivial fp32 factor
    yq = oracle.w8a8_linear_scaled_i8out(xq, wq, sx, sw, inv)
    acc = int_ref(xq, wq)
    for m in range(5):
        for n in range(9):
            # acc * 2^a * 2^b is exact in fp32 (|acc| < 2^24); then one fp32 multiply, then the rounding
            y = F32(float(Fraction(int(acc[m, n])) * Fraction(2) ** int(ex[m]) * Fraction(2) ** int(ew[n])))
            want = frac_round_half_even(Fraction(float(y * inv)))
            assert yq[m, n] == max(-127, min(127, want)), (m, n)
    assert np.abs(yq).max() == 127 and (np.abs(yq) < 127).any()  # both the saturated and the open range occur


def test_i8out_is_eq4_applied_to_the_linear_output():
    x, w = synth.w8a8_inputs(1, 12, K=512, N=48)
    xq, sx = oracle.quantize_i8_rows(x, 1e-6)
    wq, sw = oracle.quantize_i8_rows(w, 1e-6)
    exact = int_ref(xq, wq) * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    s_out = F32(np.abs(exact).max())                # static AbsMax of the layer's output
    yq = oracle.w8a8_linear_scaled_i8out(xq, wq, sx, sw, F32(127.0) / s_out)
    # X_deq = X_q / Q_8 * s is within half a step of the real output (plus three fp32 roundings)
    step = float(s_out) / 127.0
    assert np.abs(yq.astype(np.float64) * step - exact).max() <= 0.5 * step * (1 + 1e-4)
    i = np.unravel_index(np.argmax(np.abs(exact)), exact.shape)
    assert abs(int(yq[i])) == 127 and np.sign(yq[i]) == np.sign(exact[i])
    # a step that is too small saturates, symmetric, never -128
    tiny = oracle.w8a8_linear_scaled_i8out(xq, wq, sx, sw, F32(1e9))
    assert set(np.unique(tiny)).issubset({-127, 0, 127})
    # the transposed problem transposes the result
    assert np.array_equal(oracle.w8a8_linear_scaled_i8out(wq, xq, sw, sx, F32(127.0) / s_out), yq.T)
