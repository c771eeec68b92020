"""Pins for the oracle's floating-point code books (E2M1 activations, E4M3 gradients)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact import (all_finite_bf16_bits, bf16_bits_to_f64, f32_fraction, fraction_to_f32)


def bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


# the formats written out from their definition (sign, exponent field, mantissa field)
def e2m1_value(code):
    s, e, m = code >> 3, (code >> 1) & 3, code & 1
    mag = Fraction(m, 2) if e == 0 else (1 + Fraction(m, 2)) * Fraction(2) ** (e - 1)
    return -mag if s else mag


def e4m3_value(code):
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    mag = Fraction(m, 8) * Fraction(2) ** -6 if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
    return -mag if s else mag


def nearest_code(t: Fraction, negative: bool, values, sign_bit):
    """Nearest magnitude, ties to the even code, saturating; values = magnitudes by code index."""
    a = abs(t)
    best = min(range(len(values)), key=lambda i: (abs(a - values[i]), i % 2))
    return (sign_bit if negative else 0) | best


E2M1_MAGS = [e2m1_value(c) for c in range(8)]
E4M3_MAGS = [e4m3_value(c) for c in range(127)]


def unpack_fp4(codes):
    c = np.asarray(codes, np.uint8)
    out = np.empty(c.size * 2, np.uint8)
    out[0::2] = c & 0xF
    out[1::2] = c >> 4
    return out


def test_decode_tables_follow_the_format_definitions(ref):
    assert [float(v) for v in E2M1_MAGS] == [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    assert float(E4M3_MAGS[-1]) == 448.0 and float(E4M3_MAGS[1]) == 2.0 ** -9 and float(E4M3_MAGS[8]) == 2.0 ** -6
    for c in range(16):
        assert Fraction(ref.e2m1_decode(c)) == e2m1_value(c)
    assert np.signbit(np.float32(ref.e2m1_decode(8)))
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        assert Fraction(ref.e4m3_decode(c)) == e4m3_value(c)
    # library cross-check of the E4M3 table
    t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    for c in range(256):
        if c & 0x7F != 0x7F:
            assert t[c] == ref.e4m3_decode(c)


def test_encode_is_nearest_with_ties_to_even(ref):
    rng = np.random.default_rng(1)
    # E2M1: every midpoint and its float neighbours, random values, beyond the range
    pts = []
    for i in range(7):
        mid = float((E2M1_MAGS[i] + E2M1_MAGS[i + 1]) / 2)
        pts += [mid, np.nextafter(np.float32(mid), np.float32(0)), np.nextafter(np.float32(mid), np.float32(10))]
    pts += list(rng.random(400) * 6.5) + [6.0, 6.00001, 7.9, 100.0, 0.0, 1e-30]
    for t in pts:
        for sgn in (1.0, -1.0):
            v = np.float32(sgn * t)
            want = nearest_code(f32_fraction(v), bool(np.signbit(v)), E2M1_MAGS, 8)
            assert ref.e2m1_encode(v) == want, (v, want)
    assert ref.e2m1_encode(-0.0) == 8 and ref.e2m1_encode(0.0) == 0
    # E4M3: all midpoints, their neighbours, random values over the whole exponent range
    pts = []
    for i in range(126):
        mid = np.float32(float((E4M3_MAGS[i] + E4M3_MAGS[i + 1]) / 2))
        pts += [mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1000))]
    pts += list((rng.random(600) + 0.5) * 2.0 ** rng.integers(-12, 9, 600)) + [448.0, 448.1, 463.9, 1e-12]
    for t in pts:
        for sgn in (1.0, -1.0):
            v = np.float32(sgn * t)
            want = nearest_code(f32_fraction(v), bool(np.signbit(v)), E4M3_MAGS, 0x80)
            assert ref.e4m3_encode(v) == want, (v, want)
    # library cross-check: torch's own round-to-nearest-even conversion inside the finite range
    vals = ((rng.random(20000) * 2 - 1) * 448).astype(np.float32)
    vals[:2000] *= 2.0 ** -8
    got = np.array([ref.e4m3_encode(v) for v in vals], np.uint8)
    want = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, want)
    # every code survives a round trip
    assert all(ref.e2m1_encode(ref.e2m1_decode(c)) == c for c in range(16))
    assert all(ref.e4m3_encode(ref.e4m3_decode(c)) == c for c in range(256) if c & 0x7F != 0x7F)


@pytest.mark.parametrize("amax_bits", [0x3F80, 0x40C0, 0x4049, 0x3C4A, 0x0D80, 0x7149, 0x7F7F])
def test_fp4_groups_exact_over_all_bf16_patterns(ref, amax_bits):
    G = 128
    amax = float(bf16_bits_to_f64(np.array([amax_bits], np.uint16))[0])
    pats = all_finite_bf16_bits()
    pats = pats[np.abs(bf16_bits_to_f64(pats)) <= amax]
    pats = pats[:: max(1, pats.size // 6000)]                  # a spread of ~6000 patterns (rationals are slow)
    per = G - 1
    n_groups = -(-pats.size // per)
    x = np.zeros((n_groups, G), np.uint16)
    x[:, 0] = amax_bits
    x[1::2, 0] |= 0x8000
    flat = np.zeros(n_groups * per, np.uint16)
    flat[:pats.size] = pats
    x[:, 1:] = flat.reshape(n_groups, per)
    codes, scales = ref.fp4_act_quant(x, G)
    got = unpack_fp4(codes).reshape(n_groups, G)
    scale = fraction_to_f32(Fraction(amax) / 6)
    inv = fraction_to_f32(Fraction(6) / Fraction(amax))
    assert np.all(scales.view(np.uint32) == np.float32(scale).view(np.uint32))
    xv = bf16_bits_to_f64(x)
    t = (xv * np.float64(inv)).astype(np.float32)              # exact product, one rounding
    for g in range(n_groups):
        for j in range(G):
            want = nearest_code(Fraction(float(t[g, j])), bool(np.signbit(t[g, j])), E2M1_MAGS, 8)
            assert got[g, j] == want, (g, j, xv[g, j], t[g, j])
    assert np.all((got[:, 0] & 7) == 7)                        # the extreme maps to +-6
    # dequantize: exact product then bf16 rounding (torch's conversion)
    y = ref.fp4_act_dequant(codes, scales, x.size, G)
    dec = np.array([float(e2m1_value(int(c))) for c in range(16)])[got]
    dec = np.where((got & 8) != 0, -np.abs(dec), dec)          # keep -0.0
    prod = (dec * np.float64(scale)).astype(np.float32)
    assert np.array_equal(y.reshape(n_groups, G), bf16_bits(prod))


def test_fp4_dead_groups_sign_symmetry_and_error_bound(ref):
    G = 64
    x = np.zeros((3, G), np.uint16)
    x[0, ::2] = 0x8000                                         # negative zeros: still an all-zero group
    x[1, 5] = 0x0D00                                           # 2^-101
    x[2] = bf16_bits(np.random.default_rng(0).standard_normal(G).astype(np.float32))
    codes, scales = ref.fp4_act_quant(x, G)
    assert scales[0] == 0 and scales[1] == 0 and scales[2] > 0
    assert not codes[: 2 * G // 2].any()
    rng = np.random.default_rng(2)
    xb = bf16_bits(rng.standard_normal(G * 200).astype(np.float32) * 3)
    c1, s1 = ref.fp4_act_quant(xb, G)
    c2, s2 = ref.fp4_act_quant(xb ^ np.uint16(0x8000), G)
    assert np.array_equal(s1, s2) and np.array_equal(c1 ^ 0x88, c2)
    # error bound: half the spacing of the code book around the value, in scale units
    q = unpack_fp4(c1)
    xv = bf16_bits_to_f64(xb)
    dec = np.array([float(e2m1_value(int(c))) for c in range(16)])[q]
    s = np.repeat(s1.astype(np.float64), G)
    mag = np.abs(dec)
    half_gap = np.where(mag < 2, 0.25, np.where(mag < 4, 0.5, 1.0))
    assert np.all(np.abs(xv - dec * s) <= s * half_gap * (1 + 2.0 ** -18))


def test_fp8_gradient_store_against_torch_and_rationals(ref):
    rng = np.random.default_rng(3)
    G, n_groups = 128, 300
    g = (rng.standard_normal((n_groups, G)) * 1e-4).astype(np.float32)
    g[rng.random(g.shape) < 0.001] *= 100.0
    g[7] = 0.0
    g[8] = 0.0
    g[8, ::3] = -0.0
    g[9] = np.float32(1e-40)
    codes, scales = ref.fp8_grad_quant(g, G)
    amax = np.abs(g).max(axis=1)
    live = amax >= np.float32(2.0 ** -100)
    safe = np.where(live, amax, np.float32(1))
    assert np.array_equal(scales, np.where(live, safe / np.float32(448.0), 0).astype(np.float32))
    inv = np.where(live, np.float32(448.0) / safe, 0).astype(np.float32)
    t = g * inv[:, None]                                       # float32 multiply, one rounding
    want = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    want[~live] = 0                                            # dead groups: all-zero codes, sign dropped
    assert np.array_equal(codes.reshape(n_groups, G), want)
    assert not codes.reshape(n_groups, G)[7:10].any()
    assert np.all((codes.reshape(n_groups, G)[live] & 0x7F).max(axis=1) == 126)
    # plain dequantization: exact product of table value and scale
    out = ref.fp8_grad_dequant(codes, scales, G)
    table = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    assert np.array_equal(out.reshape(n_groups, G), table[codes.reshape(n_groups, G)] * scales[:, None])


@pytest.mark.parametrize("K,group,n_groups", [(1, 8, 3), (3, 8, 4), (8, 64, 2), (16, 128, 1)])
def test_fp8_reduce_matches_exact_fma_chain(ref, K, group, n_groups):
    rng = np.random.default_rng(200 + K)
    n = group * n_groups
    codes = rng.integers(0, 256, size=(K, n + group)).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x3A                       # no NaN codes
    scales = (rng.random((K, n_groups + 1)) * 1e-5 + 1e-7).astype(np.float32)
    acc = np.zeros(n, np.float32)
    for i in range(n):
        a = Fraction(0)
        for k in range(K):
            a = Fraction(float(fraction_to_f32(e4m3_value(int(codes[k, i])) * f32_fraction(scales[k, i // group]) + a)))
        acc[i] = np.float32(float(a))
    want_codes, want_scales = ref.fp8_grad_quant(acc, group)   # composition with the pinned store
    got_codes, got_scales = ref.fp8_grad_reduce_requant(codes, scales, n, group)
    assert np.array_equal(got_scales.view(np.uint32), want_scales.view(np.uint32))
    assert np.array_equal(got_codes, want_codes)


def test_fp8_reduce_uses_one_rounding_per_term(ref):
    # find inputs on which fma(v, s, acc) and acc + RN(v * s) lead to different outputs, and
    # check that the oracle follows the fused form
    table = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    rng = np.random.default_rng(11)
    group, found = 8, 0
    for _ in range(3000):
        codes = rng.integers(0, 256, size=(2, group)).astype(np.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0x41
        scales = (rng.random((2, 1)) + 0.5).astype(np.float32)
        v0, v1 = table[codes[0]], table[codes[1]]
        p0 = (v0 * scales[0, 0]).astype(np.float32)            # first term: fma(v, s, 0) = RN(v * s)
        unfused = (p0 + (v1 * scales[1, 0]).astype(np.float32)).astype(np.float32)
        fused = np.array([fraction_to_f32(f32_fraction(v1[i]) * f32_fraction(scales[1, 0]) + f32_fraction(p0[i]))
                          for i in range(group)], np.float32)
        if np.array_equal(fused, unfused):
            continue
        want = ref.fp8_grad_quant(fused, group)
        other = ref.fp8_grad_quant(unfused, group)
        if np.array_equal(want[0], other[0]) and np.array_equal(want[1], other[1]):
            continue
        found += 1
        got = ref.fp8_grad_reduce_requant(codes, scales, group, group)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
        if found >= 20:
            break
    assert found > 0


@pytest.mark.parametrize("as_bf16", [False, True])
def test_fp8_accumulate_matches_exact_arithmetic(ref, as_bf16):
    group, n = 16, 64
    rng = np.random.default_rng(77)
    codes = rng.integers(0, 256, size=n).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x22
    scales = (rng.random(n // group) * 1e-3).astype(np.float32)
    g32 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    if as_bf16:
        t = torch.from_numpy(g32).to(torch.bfloat16)
        g_in = t.view(torch.int16).numpy().view(np.uint16)
        g32 = t.to(torch.float32).numpy()
    else:
        g_in = g32
    acc = np.array([fraction_to_f32(e4m3_value(int(codes[i])) * f32_fraction(scales[i // group]) + f32_fraction(g32[i]))
                    for i in range(n)], np.float32)
    want = ref.fp8_grad_quant(acc, group)
    got = ref.fp8_grad_accumulate(codes, scales, g_in, group)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
    # accumulating onto an all-zero stored gradient is the plain store
    z = ref.fp8_grad_accumulate(np.zeros(n, np.uint8), np.zeros(n // group, np.float32), g_in, group)
    plain = ref.fp8_grad_quant(g32, group)
    assert np.array_equal(z[0], plain[0]) and np.array_equal(z[1], plain[1])


def test_fp8_accumulate_uses_one_rounding(ref):
    table = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    rng = np.random.default_rng(12)
    group, found = 8, 0
    for _ in range(4000):
        codes = rng.integers(0, 256, size=group).astype(np.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0x41
        scale = (rng.random(1) + 0.5).astype(np.float32)
        g = (rng.standard_normal(group) * 50).astype(np.float32)
        v = table[codes]
        unfused = ((v * scale[0]).astype(np.float32) + g).astype(np.float32)
        fused = np.array([fraction_to_f32(f32_fraction(v[i]) * f32_fraction(scale[0]) + f32_fraction(g[i]))
                          for i in range(group)], np.float32)
        if np.array_equal(fused, unfused):
            continue
        want, other = ref.fp8_grad_quant(fused, group), ref.fp8_grad_quant(unfused, group)
        if np.array_equal(want[0], other[0]) and np.array_equal(want[1], other[1]):
            continue
        found += 1
        got = ref.fp8_grad_accumulate(codes, scale, g, group)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
        if found >= 10:
            break
    assert found > 0
