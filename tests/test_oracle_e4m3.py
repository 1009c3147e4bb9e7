"""Pins for the oracle's bf16 / E4M3 / amax / scale / quantize functions (CPU only).

Each check compares the oracle with something that is not the oracle: the
range the paper prints, a table built from exact rationals, a brute-force
nearest-value search, a library cast, or a textbook definition.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2511_23225_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_constants():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def exact_table():
    """All finite E4M3 values as exact rationals, built from the format definition."""
    vals = {}
    for b in range(256):
        s, e, m = b >> 7, (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            continue
        if e == 0:
            v = Fraction(m, 8) * Fraction(1, 64)
        else:
            v = (1 + Fraction(m, 8)) * (Fraction(2) ** (e - 7))
        vals[b] = -v if s else v
    return vals


TABLE = exact_table()
POS = sorted((v, b) for b, v in TABLE.items() if b < 0x80)


def brute_encode(v):
    """Nearest finite E4M3 value in exact arithmetic; ties -> even mantissa; saturate."""
    if v != v:
        return None
    sign = 0x80 if np.signbit(np.float32(v)) else 0
    if np.isinf(v):
        return sign | 0x7E
    a = abs(Fraction(float(v)))
    if a >= 448:
        return sign | 0x7E
    best = None
    for val, code in POS:
        d = abs(val - a)
        if best is None or d < best[0] or (d == best[0] and (code & 1) == 0):
            best = (d, code)
    return sign | best[1]


def test_range_is_paper_value():
    c = paper_constants()
    finite = [float(v) for v in TABLE.values()]
    assert max(finite) == c["e4m3_max"] == 448.0
    assert min(finite) == -448.0
    assert oracle.e4m3_decode(0x7E) == 448.0 and oracle.e4m3_decode(0xFE) == -448.0
    assert np.isnan(oracle.e4m3_decode(0x7F)) and np.isnan(oracle.e4m3_decode(0xFF))


def test_decode_matches_exact_table_and_spacing():
    for b, v in TABLE.items():
        assert Fraction(oracle.e4m3_decode(b)) == v
    # spacing doubles every 8 codes above the subnormal band; 126 positive finite codes
    pos = [v for v, _ in POS]
    assert len(pos) == 127 and pos[0] == 0 and pos[1] == Fraction(1, 512)
    for i in range(1, 16):
        gap = pos[8 * i + 1] - pos[8 * i] if 8 * i + 1 < len(pos) else None
        if gap is not None:
            assert gap == Fraction(2) ** (max(i, 1) - 7 - 3)


def test_decode_matches_library_dtype():
    codes = torch.arange(256, dtype=torch.uint8)
    lib_vals = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for b in range(256):
        o = oracle.e4m3_decode(b)
        if np.isnan(o):
            assert np.isnan(lib_vals[b])
        else:
            assert o == lib_vals[b]


def test_encode_roundtrip_all_codes():
    for b in TABLE:
        assert oracle.e4m3_encode(oracle.e4m3_decode(b)) == b


def test_encode_midpoints_and_neighbours():
    pos = [float(v) for v, _ in POS]
    for i in range(len(pos) - 1):
        lo, hi = np.float32(pos[i]), np.float32(pos[i + 1])
        mid = np.float32((float(lo) + float(hi)) / 2)  # exact in fp32
        assert float(mid) * 2 == float(lo) + float(hi)
        for v in (mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)), lo, hi):
            for sgn in (1.0, -1.0):
                x = np.float32(sgn) * v
                assert oracle.e4m3_encode(x) == brute_encode(x), (x, i)
    # the tie at exactly 2^-10 (half the smallest subnormal) goes to even = 0
    assert oracle.e4m3_encode(2.0 ** -10) == 0
    assert oracle.e4m3_encode(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 1
    assert oracle.e4m3_encode(-0.0) == 0x80


def test_encode_brute_force_random_and_edges():
    rng = np.random.default_rng(7)
    vals = np.concatenate([
        rng.standard_normal(3000).astype(np.float32),
        (rng.standard_normal(3000) * 200).astype(np.float32),
        (rng.standard_normal(2000) * 0.01).astype(np.float32),
        np.exp(rng.uniform(np.log(1e-5), np.log(2e3), 3000)).astype(np.float32),
        np.array([0, 447.99, 448, 463.9, 464, 480, 1e4, 3e38, np.inf, -np.inf, 1e-30, 1.4e-45],
                 np.float32),
    ])
    for v in vals:
        assert oracle.e4m3_encode(v) == brute_encode(v), v
    assert oracle.e4m3_encode(np.nan) & 0x7F == 0x7F


def test_encode_is_monotone():
    grid = np.sort(np.concatenate([np.linspace(-500, 500, 20001), np.linspace(-0.05, 0.05, 20001)])
                   .astype(np.float32))
    prev = -1e9
    for v in grid:
        d = oracle.e4m3_decode(oracle.e4m3_encode(v))
        assert d >= prev
        prev = d


def test_encode_matches_library_cast_in_range():
    # torch's float8_e4m3fn cast rounds to nearest even but does not saturate; it
    # agrees with a saturating cast for |v| <= 464.
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.uniform(-464, 464, 20000), rng.standard_normal(20000) * 0.02,
                        rng.standard_normal(20000)]).astype(np.float32)
    lib_codes = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([oracle.e4m3_encode(x) for x in v], np.uint8)
    assert np.array_equal(lib_codes, mine)


def test_bf16_helpers():
    allh = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = oracle.bf16_to_f32(allh)
    ref = torch.from_numpy(allh.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(f.view(np.uint32), ref.view(np.uint32))
    # round trip of every non-NaN pattern, ties to even, against the library's cast
    for h in list(range(0, 65536, 97)) + [0x7F7F, 0x7F80, 0xFF80, 0x0001, 0x8000]:
        x = f[h]
        if not np.isnan(x):
            assert oracle.f32_to_bf16_scalar(x) == h
    rng = np.random.default_rng(3)
    u = rng.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32)
    u = np.concatenate([u, np.array([0x3F808000, 0x3F818000, 0x3F80FFFF, 0x7F7FFFFF, 0x00008000],
                                    np.uint32)])
    x = u.view(np.float32)
    lib_bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for xi, lb in zip(x, lib_bits):
        if not np.isnan(xi):
            assert oracle.f32_to_bf16_scalar(xi) == lb
    assert oracle.f32_to_bf16_scalar(np.float32(np.nan)) & 0x7FFF > 0x7F80


def test_amax_textbook_and_edges():
    rng = np.random.default_rng(5)
    x = synth.f32_to_bf16_bits(rng.standard_normal(10007).astype(np.float32) * 37)
    assert oracle.amax_bf16(x) == np.max(np.abs(synth.bf16_bits_to_f32(x)))
    assert oracle.amax_bf16(rng.permutation(x)) == oracle.amax_bf16(x)
    assert oracle.amax_bf16(np.zeros(5, np.uint16)) == 0.0
    assert oracle.amax_bf16(np.array([0xC2F7], np.uint16)) == synth.bf16_bits_to_f32([0x42F7])[0]
    assert np.isinf(oracle.amax_bf16(np.array([0x3F80, 0xFF80, 0x4000], np.uint16)))
    assert np.isnan(oracle.amax_bf16(np.array([0x3F80, 0x7F80, 0x7FC0], np.uint16)))


def test_scale_definition_and_guards():
    for amax in (448.0, 896.0, 1.0, 0.013, 9873.0, 3.2e4):
        s, si = oracle.scale_from_amax(np.float32(amax))
        assert s == np.float32(448.0) / np.float32(amax)
        assert si == np.float32(1.0) / s
    assert oracle.scale_from_amax(448.0) == (1.0, 1.0)
    assert oracle.scale_from_amax(448.0 * 8)[0] == 0.125
    for bad in (0.0, np.inf, np.nan):
        assert oracle.scale_from_amax(bad) == (1.0, 1.0)
    s, si = oracle.scale_from_amax(np.float32(1e-42))
    assert np.isfinite(s) and s == np.finfo(np.float32).max


def test_quantize_composition_transpose_and_amax_saturates():
    x, _, _ = synth.fp8_linear_inputs(0, 0)
    amax = oracle.amax_bf16(x)
    assert 1000 <= amax <= 10000  # the injected extreme outliers set the scale (Sec. 1)
    scale, _ = oracle.scale_from_amax(amax)
    q, qT = oracle.quantize_e4m3(x, scale)
    assert np.array_equal(qT, q.T)
    # independent recomputation: numpy fp32 multiply + the brute-force encoder on a sample
    prod = synth.bf16_bits_to_f32(x) * np.float32(scale)
    rng = np.random.default_rng(1)
    for i in rng.integers(0, x.size, 3000):
        r, c = divmod(int(i), x.shape[1])
        assert q[r, c] == brute_encode(prod[r, c])
    # elements attaining amax land on +-448
    top = (x & 0x7FFF) == (x & 0x7FFF).max()
    assert set((q[top] & 0x7F).tolist()) == {0x7E}
    # the workload exercises flush-to-zero, subnormal, normal and saturating codes
    mag = q & 0x7F
    assert (mag == 0).mean() > 0.005 and ((mag > 0) & (mag < 8)).mean() > 0.1
    assert (mag >= 8).mean() > 0.3 and (mag == 0x7E).sum() >= 1
    # scale 1 (amax 448) reduces quantize to the plain encoder
    x2 = x.copy()
    x2[0, 0] = 0x43E0  # 448.0
    x2[(x2 & 0x7FFF) > 0x43E0] = 0x3F80
    assert oracle.scale_from_amax(oracle.amax_bf16(x2))[0] == 1.0
    q2, _ = oracle.quantize_e4m3(x2[:4], 1.0)
    f2 = synth.bf16_bits_to_f32(x2[:4])
    assert all(q2[r, c] == brute_encode(f2[r, c]) for r in range(4) for c in range(0, 512, 7))


def test_quantize_subnormal_fp32_products_are_honoured():
    # products below the fp32 normal range must not be flushed before rounding
    x = np.array([[0x0080, 0x0001, 0x8001, 0x0100]], np.uint16)  # tiny bf16 values
    q, _ = oracle.quantize_e4m3(x, np.float32(0.5), transpose=False)
    assert q.tolist() == [[0, 0, 0x80, 0]]
    q, _ = oracle.quantize_e4m3(x, np.finfo(np.float32).max, transpose=False)
    f = synth.bf16_bits_to_f32(x) * np.finfo(np.float32).max
    assert q.tolist() == [[brute_encode(v) for v in f[0]]]


# ------------------------------------------------------------ delayed scaling (Sec. 4.3)


def _tensor_with_amax(amax, seed, shape=(16, 32)):
    rng = np.random.default_rng(seed)
    v = (rng.uniform(-0.5, 0.5, shape) * amax).astype(np.float32)
    v[0, 0] = amax
    return synth.f32_to_bf16_bits(v)


def test_delayed_scaling_window_of_sixteen():
    # what the recipe fixes: the scale of a step comes from the amax values of up to 16 earlier
    # steps and never from the tensor itself (except on an empty history)
    d = oracle.DelayedScaling()
    amaxes = [2.0] * 3 + [512.0] + [2.0] * 20
    used = []
    for t, a in enumerate(amaxes):
        q, qT, s, si = d.cast(_tensor_with_amax(a, t))
        used.append(float(s))
        assert np.array_equal(qT, q.T)
        assert np.float32(si) == np.float32(1.0) / np.float32(s)
    assert used[0] == 448.0 / 2.0                      # bootstrap: own amax
    assert used[1] == used[2] == used[3] == 448.0 / 2.0  # the spike at step 3 is cast with the old scale
    assert all(u == 448.0 / 512.0 for u in used[4:20])  # ... and then rules the next 16 steps
    assert all(u == 448.0 / 2.0 for u in used[20:])      # and is forgotten afterwards
    assert len(d.history) == 16


def test_delayed_scaling_saturates_what_the_old_scale_cannot_hold():
    # the paper's point about this recipe: a spike the history has not seen overflows the format
    d = oracle.DelayedScaling()
    d.cast(_tensor_with_amax(1.0, 0))
    x = _tensor_with_amax(64.0, 1)
    q, _, s, _ = d.cast(x)
    assert float(s) == 448.0
    vals = synth.bf16_bits_to_f32(x).astype(np.float64) * 448.0
    assert np.all((q[np.abs(vals) >= 448.0] & 0x7F) == 0x7E)   # saturated, never the NaN code
    assert np.array_equal(q, oracle.quantize_e4m3(x, np.float32(448.0))[0])


def test_delayed_scaling_bootstrap_is_current_scaling():
    x, _, _ = synth.fp8_linear_inputs(0, 0)
    d = oracle.DelayedScaling()
    q, qT, s, si = d.cast(x)
    s_ref, si_ref = oracle.scale_from_amax(oracle.amax_bf16(x))
    assert s == s_ref and si == si_ref
    assert np.array_equal(q, oracle.quantize_e4m3(x, s_ref)[0])
