"""Pins for the oracle's LayerNorm, residual add and fp64 -> bf16 rounding (CPU only).

The paper (Sec. 4.3) only says that the LayerNorm components run under FP8 together with the
linear layers; the normalisation itself is the textbook one, so the pins are closed forms,
invariances, exact rational arithmetic and a library routine."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2511_23225_amd import synth

ONE = synth.f32_to_bf16_bits(np.ones(1, np.float32))[0]


def bits(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def val(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


def bf16_value(p):
    """Exact rational value of a finite bf16 pattern, from the format definition."""
    s, e, m = p >> 15, (p >> 7) & 0xFF, p & 0x7F
    assert e != 0xFF
    v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -v if s else v


def test_f64_to_bf16_brute_force_against_the_value_grid():
    # nearest bf16 value in exact rationals, ties to the even pattern, around every kind of place:
    # random values, exact midpoints and their fp64 neighbours, subnormals, the overflow edge
    rng = np.random.default_rng(1)
    pats = np.concatenate([rng.integers(0, 0x7F7F, 300), [0, 1, 2, 0x7F, 0x80, 0x81, 0x7F7E]]).astype(int)
    for p in pats:
        lo, hi = bf16_value(int(p)), bf16_value(int(p) + 1)
        mid = (lo + hi) / 2
        fm = float(mid)  # midpoints of adjacent bf16 values are exact in fp64
        assert Fraction(fm) == mid
        want_tie = int(p) if int(p) % 2 == 0 else int(p) + 1
        assert oracle.f64_to_bf16_scalar(fm) == want_tie
        assert oracle.f64_to_bf16_scalar(np.nextafter(fm, 0.0)) == int(p)
        assert oracle.f64_to_bf16_scalar(np.nextafter(fm, np.inf)) == int(p) + 1
        assert oracle.f64_to_bf16_scalar(-fm) == (want_tie | 0x8000)
        assert oracle.f64_to_bf16_scalar(float(lo)) == int(p)
    top = float(bf16_value(0x7F7F))
    assert oracle.f64_to_bf16_scalar(top) == 0x7F7F
    tie = top + 2.0 ** 119                                 # half an ulp (2^120) above the largest finite value
    assert oracle.f64_to_bf16_scalar(tie) == 0x7F80        # the tie goes to the even pattern: Inf
    assert oracle.f64_to_bf16_scalar(np.nextafter(tie, 0.0)) == 0x7F7F
    assert oracle.f64_to_bf16_scalar(float("inf")) == 0x7F80 and oracle.f64_to_bf16_scalar(-0.0) == 0x8000
    assert oracle.f64_to_bf16_scalar(float("nan")) & 0x7FFF > 0x7F80


def test_f64_to_bf16_agrees_with_the_fp32_routine_and_a_library_cast():
    # for values that are exactly fp32 the single rounding equals the fp32 -> bf16 rounding
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-30, 30, 4000), [0.0, 1.0, -3.0]])
    v = v.astype(np.float32)
    got = np.array([oracle.f64_to_bf16_scalar(float(x)) for x in v], np.uint16)
    lib_cast = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, lib_cast)
    assert np.array_equal(got, synth.f32_to_bf16_bits(v))
    # and it avoids the double rounding a detour through fp32 makes: 1 + 2^-8 + 2^-40 is above the tie
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert oracle.f64_to_bf16_scalar(x) == ONE + 1
    assert synth.f32_to_bf16_bits(np.float32(x).reshape(1))[0] == ONE  # fp32 first: falls on the tie, goes to even


def test_residual_add_is_the_exact_sum_rounded_once():
    rng = np.random.default_rng(3)
    x = bits(rng.standard_normal(5000) * 3)
    r = bits(rng.standard_normal(5000) * 100)
    h = oracle.residual_add_bf16(x, r)
    for i in range(0, 5000, 7):
        exact = bf16_value(int(x[i])) + bf16_value(int(r[i]))
        hv = bf16_value(int(h[i]))
        # nearest: no other bf16 value is closer
        for nb in (int(h[i]) - 1, int(h[i]) + 1):
            if 0 <= (nb & 0x7FFF) < 0x7F80 and (nb >> 15) == (int(h[i]) >> 15) and nb >= 0:
                assert abs(hv - exact) <= abs(bf16_value(nb) - exact)
    # library: the fp32 sum of two bf16 values is exact here (exponents close), torch rounds it once
    x2, r2 = bits(rng.standard_normal(5000)), bits(rng.standard_normal(5000))
    want = (torch.from_numpy(val(x2) + val(r2)).to(torch.float32).to(torch.bfloat16)
            .view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(oracle.residual_add_bf16(x2, r2), want)


def test_layernorm_constant_row_gives_beta():
    cols = 96
    h = bits(np.full((2, cols), 5.5))
    gamma = bits(np.linspace(0.5, 2.0, cols))
    beta = bits(np.linspace(-1.0, 1.0, cols))
    y64, yb = oracle.layernorm(h, gamma, beta, eps=1e-5)
    assert np.array_equal(y64, np.broadcast_to(val(beta), (2, cols)))   # (h - mu) = 0 exactly
    assert np.array_equal(yb, np.broadcast_to(beta, (2, cols)))
    y64, _ = oracle.layernorm(h, gamma, None, eps=1e-5)
    assert np.all(y64 == 0.0)


def test_layernorm_two_valued_row_closed_form():
    # half of the row at a, half at b: mu = (a+b)/2, var = ((a-b)/2)^2, so the normalised values are
    # +-d / sqrt(d^2 + eps) with d = (a-b)/2, times gamma, plus beta
    cols = 64
    a, b, eps = 3.0, -1.0, 1e-3
    row = np.where(np.arange(cols) % 2 == 0, a, b)
    gamma = bits(np.full(cols, 1.5))
    beta = bits(np.full(cols, 0.25))
    y64, yb = oracle.layernorm(bits(row[None, :]), gamma, beta, eps)
    d = (a - b) / 2
    want = np.where(np.arange(cols) % 2 == 0, 1.0, -1.0) * d / np.sqrt(d * d + eps) * 1.5 + 0.25
    assert np.allclose(y64[0], want, rtol=1e-15, atol=0)
    assert np.array_equal(yb[0], np.array([oracle.f64_to_bf16_scalar(w) for w in want], np.uint16))


def test_layernorm_unit_gamma_zero_beta_moments():
    rng = np.random.default_rng(4)
    rows, cols, eps = 7, 768, 1e-5
    h = bits(rng.standard_normal((rows, cols)) * 4 + 2)
    y64, _ = oracle.layernorm(h, np.full(cols, ONE, np.uint16), None, eps)
    hv = val(h)
    var = hv.var(axis=1)                       # numpy's biased variance
    assert np.allclose(y64.mean(axis=1), 0.0, atol=1e-14)
    assert np.allclose((y64 ** 2).mean(axis=1), var / (var + eps), rtol=1e-13)


def test_layernorm_shift_and_scale_invariance():
    rng = np.random.default_rng(5)
    cols = 256
    base = np.round(rng.standard_normal((3, cols)) * 8) / 8     # multiples of 1/8, |.| < 8: exact in bf16
    gamma, beta = bits(rng.standard_normal(cols)), bits(rng.standard_normal(cols))
    y0, _ = oracle.layernorm(bits(base), gamma, beta, 1e-5)
    y1, _ = oracle.layernorm(bits(base + 16.0), gamma, beta, 1e-5)      # still exact in bf16
    assert np.allclose(y0, y1, rtol=1e-13, atol=1e-13)
    y2, _ = oracle.layernorm(bits(base * 4.0), gamma, beta, 16 * 1e-5)  # (4h, 16 eps) is the same map
    assert np.allclose(y0, y2, rtol=1e-13, atol=1e-13)
    # a swapped sign or a dropped beta would show here
    y3, _ = oracle.layernorm(bits(-base), gamma, beta, 1e-5)
    assert np.allclose(y3 - val(beta), -(y0 - val(beta)), rtol=1e-13, atol=1e-13)


def test_layernorm_exact_rationals_tiny():
    # y^2 (var + eps) = (h - mu)^2 gamma^2 holds in exact rationals up to the fp64 rounding of y
    rng = np.random.default_rng(6)
    cols = 5
    h = bits(rng.standard_normal((2, cols)) * 3)
    gamma = bits(rng.standard_normal(cols))
    eps = 2.0 ** -10
    y64, _ = oracle.layernorm(h, gamma, None, eps)
    for r in range(2):
        H = [bf16_value(int(p)) for p in h[r]]
        mu = sum(H) / cols
        var = sum((x - mu) ** 2 for x in H) / cols
        for c in range(cols):
            lhs = Fraction(float(y64[r, c])) ** 2 * (var + Fraction(eps))
            rhs = (H[c] - mu) ** 2 * bf16_value(int(gamma[c])) ** 2
            assert abs(lhs - rhs) <= rhs * Fraction(1, 2 ** 48)
            assert (y64[r, c] > 0) == ((H[c] - mu) * bf16_value(int(gamma[c])) > 0)


def test_layernorm_against_a_library_in_fp64():
    rng = np.random.default_rng(7)
    for rows, cols, eps in ((5, 768, 1e-5), (3, 2048, 1e-6), (4, 200, 1e-5)):
        h = bits(rng.standard_normal((rows, cols)) * 5)
        h[0, 3] = bits(np.float32(3000.0).reshape(1))[0]            # an extreme outlier in a row
        gamma, beta = bits(1 + 0.1 * rng.standard_normal(cols)), bits(0.1 * rng.standard_normal(cols))
        y64, yb = oracle.layernorm(h, gamma, beta, eps)
        want = torch.nn.functional.layer_norm(torch.from_numpy(val(h)), (cols,), torch.from_numpy(val(gamma)),
                                              torch.from_numpy(val(beta)), eps).numpy()
        assert np.allclose(y64, want, rtol=1e-12, atol=1e-13)
        # the stored activation is the single rounding of the fp64 value
        sample = [(0, 3), (1, 17), (rows - 1, cols - 1)]
        for r, c in sample:
            assert yb[r, c] == oracle.f64_to_bf16_scalar(y64[r, c])
