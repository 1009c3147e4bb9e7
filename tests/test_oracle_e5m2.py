"""Pins for the oracle's E5M2 functions (the gradient format of the paper's HYBRID recipe, Sec. 4.3),
CPU only: exact rationals built from the format definition, a brute-force nearest-value search,
the library dtype, and exact-rational GEMMs on tiny shapes."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2511_23225_amd import synth


def exact_table():
    vals = {}
    for b in range(256):
        s, e, m = b >> 7, (b >> 2) & 31, b & 3
        if e == 31:
            continue  # Inf / NaN codes
        v = Fraction(m, 4) * Fraction(1, 2 ** 14) if e == 0 else (1 + Fraction(m, 4)) * Fraction(2) ** (e - 15)
        vals[b] = -v if s else v
    return vals


TABLE = exact_table()
POS = sorted((v, b) for b, v in TABLE.items() if b < 0x80)


def brute_encode(v):
    sign = 0x80 if np.signbit(np.float32(v)) else 0
    if np.isinf(v):
        return sign | 0x7B
    a = abs(Fraction(float(v)))
    if a >= 57344:
        return sign | 0x7B
    best = None
    for val, code in POS:
        d = abs(val - a)
        if best is None or d < best[0] or (d == best[0] and code % 2 == 0 and best[1] % 2 == 1):
            best = (d, code)
    return sign | best[1]


def test_decode_matches_exact_table_and_library_dtype():
    for b, v in TABLE.items():
        assert Fraction(oracle.e5m2_decode(b)) == v, hex(b)
    assert oracle.e5m2_decode(0x7B) == 57344.0 and oracle.e5m2_decode(0xFB) == -57344.0  # largest finite
    assert oracle.e5m2_decode(0x01) == 2.0 ** -16  # smallest subnormal
    assert np.isinf(oracle.e5m2_decode(0x7C)) and np.isnan(oracle.e5m2_decode(0x7D))
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).to(torch.float32).numpy()
    for b in range(256):
        d = oracle.e5m2_decode(b)
        assert (np.isnan(d) and np.isnan(lib[b])) or d == lib[b], hex(b)


def test_encode_roundtrip_midpoints_and_saturation():
    for b in TABLE:
        if b & 0x7F:  # -0 and +0 keep their sign
            assert oracle.e5m2_encode(oracle.e5m2_decode(b)) == b, hex(b)
    assert oracle.e5m2_encode(0.0) == 0x00 and oracle.e5m2_encode(-0.0) == 0x80
    # every midpoint between neighbouring values and its two fp32 neighbours
    for (lo, cl), (hi, ch) in zip(POS[:-1], POS[1:]):
        mid = np.float32(float((lo + hi) / 2))
        assert Fraction(float(mid)) == (lo + hi) / 2  # exactly representable in fp32
        for v in (np.nextafter(mid, np.float32(0)), mid, np.nextafter(mid, np.float32(np.inf))):
            assert oracle.e5m2_encode(v) == brute_encode(v), (float(v), cl, ch)
            assert oracle.e5m2_encode(-v) == (brute_encode(v) | 0x80)
    for v in (57344.0, 57345.0, 61439.9, 61440.0, 65536.0, 1e30, np.inf):
        assert oracle.e5m2_encode(v) == 0x7B and oracle.e5m2_encode(-v) == 0xFB
    assert oracle.e5m2_encode(np.nan) & 0x7F in (0x7D, 0x7E, 0x7F)


def test_encode_brute_force_random_and_monotone():
    rng = np.random.default_rng(5)
    vals = np.concatenate([rng.standard_normal(3000) * s for s in (1e-5, 1e-3, 1.0, 100.0, 3e4)]).astype(np.float32)
    for v in vals:
        assert oracle.e5m2_encode(v) == brute_encode(v), float(v)
    grid = np.sort(np.abs(vals))
    codes = [oracle.e5m2_encode(v) for v in grid]
    assert all(a <= b for a, b in zip(codes[:-1], codes[1:]))


def test_encode_matches_library_cast_in_range():
    rng = np.random.default_rng(6)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-12, 10, 20000))).astype(np.float32)
    v = v[np.abs(v) < 57344.0]
    lib = torch.from_numpy(v).to(torch.float8_e5m2).view(torch.uint8).numpy()
    ours = np.array([oracle.e5m2_encode(x) for x in v], dtype=np.uint8)
    assert np.array_equal(ours, lib)


def test_scale_and_quantize_e5m2():
    s, si = oracle.scale_from_amax_e5m2(57344.0)
    assert s == 1.0 and si == 1.0
    s, si = oracle.scale_from_amax_e5m2(2.0 ** -3 * 57344.0)
    assert s == 8.0 and si == 0.125
    for bad in (0.0, np.inf, np.nan):
        assert oracle.scale_from_amax_e5m2(bad) == (1.0, 1.0)
    rng = np.random.default_rng(7)
    x = torch.from_numpy(rng.standard_normal((24, 40)).astype(np.float32)).to(torch.bfloat16)
    bits = x.view(torch.int16).numpy().view(np.uint16)
    amax = float(x.abs().max())
    s, _ = oracle.scale_from_amax_e5m2(amax)
    q, qT = oracle.quantize_e5m2(bits, s)
    assert np.array_equal(qT, q.T)
    assert (q.max() & 0x7F) == 0x7B or (q[np.unravel_index(np.argmax(np.abs(x.float().numpy())), q.shape)] & 0x7F) == 0x7B
    prod = (x.float().numpy() * np.float32(s)).astype(np.float32)
    want = np.array([[brute_encode(v) for v in row] for row in prod], dtype=np.uint8)
    assert np.array_equal(q, want)


def test_gradient_gemms_with_e5m2_dy_match_exact_rationals():
    rng = np.random.default_rng(8)
    M, N, K = 3, 5, 4
    e4 = {}
    for b in range(256):
        sgn, e, m = b >> 7, (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            continue
        v = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        e4[b] = -v if sgn else v
    dyq = rng.choice(sorted(TABLE), size=(M, N)).astype(np.uint8)
    wq = rng.choice(sorted(e4), size=(N, K)).astype(np.uint8)
    xq = rng.choice(sorted(e4), size=(M, K)).astype(np.uint8)
    sdy, sw, sx = np.float32(0.75), np.float32(1.5), np.float32(0.3125)
    dx, _ = oracle.fp8_linear_dgrad(dyq, wq, sdy, sw, dy_e5m2=True)
    dw, _ = oracle.fp8_linear_wgrad(dyq, xq, sdy, sx, dy_e5m2=True)
    for m in range(M):
        for k in range(K):
            ex = sum(TABLE[int(dyq[m, n])] * e4[int(wq[n, k])] for n in range(N)) * Fraction(float(sdy)) * Fraction(float(sw))
            assert abs(dx[m, k] - float(ex)) <= 1e-12 * max(1.0, abs(float(ex)))
    for n in range(N):
        for k in range(K):
            ex = sum(TABLE[int(dyq[m, n])] * e4[int(xq[m, k])] for m in range(M)) * Fraction(float(sdy)) * Fraction(float(sx))
            assert abs(dw[n, k] - float(ex)) <= 1e-12 * max(1.0, abs(float(ex)))


def _tensor_with_amax(amax, seed, shape=(16, 32)):
    rng = np.random.default_rng(seed)
    v = (rng.uniform(-0.5, 0.5, shape) * amax).astype(np.float32)
    v[0, 0] = amax
    return synth.f32_to_bf16_bits(v)


def test_delayed_scaling_with_e5m2_gradients():
    # HYBRID + delayed scaling as the paper ran it (Sec. 4.3): the same 16-deep window, the scale
    # maps into +-57344, the bytes are E5M2 codes of x * scale
    d = oracle.DelayedScaling(e5m2=True)
    amaxes = [2.0] * 3 + [512.0] + [2.0] * 20
    used = []
    for t, a in enumerate(amaxes):
        x = _tensor_with_amax(a, t)
        q, qT, s, si = d.cast(x)
        used.append(float(s))
        assert np.array_equal(qT, q.T)
        assert np.float32(si) == np.float32(1.0) / np.float32(s)
        assert np.array_equal(q, oracle.quantize_e5m2(x, np.float32(s))[0])
    assert used[0] == used[1] == used[2] == used[3] == 57344.0 / 2.0
    assert all(u == 57344.0 / 512.0 for u in used[4:20]) and all(u == 57344.0 / 2.0 for u in used[20:])
    # a spike the history has not seen saturates at the largest finite code, never inf
    d = oracle.DelayedScaling(e5m2=True)
    d.cast(_tensor_with_amax(1.0, 0))
    q, _, s, _ = d.cast(_tensor_with_amax(64.0, 1))
    assert float(s) == 57344.0 and (q[0, 0] & 0x7F) == 0x7B and not ((q & 0x7F) == 0x7C).any()
