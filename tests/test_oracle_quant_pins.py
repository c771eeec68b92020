"""Pins for the oracle's quantize / dequantize arithmetic (CPU only).

The paper prints no worked numeric example of its block-wise quantizer, so the
oracle is pinned by what the mathematics fixes: exact rational arithmetic over
every bf16 bit pattern, closed forms on power-of-two scales, tie cases,
invariants, byte-level packing fixtures and library cross-checks.
"""
from fractions import Fraction
import os

import numpy as np
import pytest
import torch

from exact import (all_finite_bf16_bits, bf16_bits_to_f64, bf16_rne_from_fraction,
                   f32_fraction, fraction_to_f32, pack_codes, rint_half_even_f64, unpack_codes)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_bits(x):
    """fp32 array -> bf16 bit patterns through torch (library conversion)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


ALL_BITS = [4, 5, 6, 8]


def codes_to_int(codes, bits):
    codes = np.asarray(codes, np.uint8)
    return unpack_codes(codes, codes.size * 8 // bits, bits)


# ---------------------------------------------------------------------------
# exact-arithmetic brute force over every bf16 pattern below a planted amax
# ---------------------------------------------------------------------------

PLANTED_AMAX_BITS = [
    0x3F80,  # 1.0
    0x40E0,  # 7.0      (4-bit scale exactly 1)
    0x42FE,  # 127.0    (8-bit scale exactly 1)
    0x4049,  # 3.140625
    0x3FFF,  # 1.9921875 (largest significand)
    0x3C4A,  # ~0.0123
    0x1280,  # ~8.08e-28
    0x0D80,  # 2^-100   (smallest amax that is still quantized)
    0x7149,  # ~9.96e29
    0x7F7F,  # largest finite bf16
]


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("amax_bits", PLANTED_AMAX_BITS)
def test_codes_and_scale_exact_all_bf16_patterns(ref, bits, amax_bits):
    G = 128
    qmax = (1 << (bits - 1)) - 1
    amax = float(bf16_bits_to_f64(np.array([amax_bits], np.uint16))[0])
    pats = all_finite_bf16_bits()
    vals = bf16_bits_to_f64(pats)
    pats = pats[np.abs(vals) <= amax]
    # groups of G: element 0 is +-amax (alternating), the rest are the patterns
    per = G - 1
    n_groups = -(-pats.size // per)
    x = np.zeros((n_groups, G), np.uint16)
    x[:, 0] = amax_bits
    x[1::2, 0] |= 0x8000
    flat = np.zeros(n_groups * per, np.uint16)
    flat[:pats.size] = pats
    x[:, 1:] = flat.reshape(n_groups, per)

    codes, scales = ref.act_quant(x, G, bits)
    got = codes_to_int(codes, bits).reshape(n_groups, G)

    # expected, from rationals: scale = RN(amax/qmax), inv = RN(qmax/amax)
    scale = fraction_to_f32(Fraction(amax) / qmax)
    inv = fraction_to_f32(Fraction(qmax) / Fraction(amax))
    assert np.all(scales.view(np.uint32) == np.float32(scale).view(np.uint32))
    # t = RN32(x * inv): the product of two binary32 values is exact in binary64
    xv = bf16_bits_to_f64(x)
    t = (xv * np.float64(inv)).astype(np.float32)
    want = np.clip(rint_half_even_f64(t.astype(np.float64)), -qmax, qmax).astype(np.int32)
    assert np.array_equal(got, want)
    # the planted extreme maps to +-qmax exactly, nothing exceeds it
    assert np.all(np.abs(got[:, 0]) == qmax)
    assert np.abs(got).max() == qmax


def test_exact_helper_agrees_with_fraction_products():
    # the float64 shortcut above is itself checked against pure rationals
    rng = np.random.default_rng(5)
    for _ in range(300):
        a = np.float32(rng.standard_normal() * 10.0 ** rng.integers(-20, 20))
        b = np.float32(rng.standard_normal() * 10.0 ** rng.integers(-15, 15))
        want = fraction_to_f32(f32_fraction(a) * f32_fraction(b))
        got = np.float32(np.float64(a) * np.float64(b))
        assert got.view(np.uint32) == want.view(np.uint32)
        assert (a * b).view(np.uint32) == want.view(np.uint32)


# ---------------------------------------------------------------------------
# tie cases on a power-of-two scale: half-even, not half-away, not truncation
# ---------------------------------------------------------------------------

def load_tie_fixture():
    rows = []
    with open(os.path.join(GOLDEN, "rint_ties.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                t, q = line.split()
                rows.append((float(t), int(q)))
    return rows


@pytest.mark.parametrize("bits", ALL_BITS)
def test_ties_round_to_even(ref, bits):
    qmax = (1 << (bits - 1)) - 1
    # keep the rows that fit the grid and that bf16 (8 significant bits) can hold
    rows = [(t, q) for t, q in load_tie_fixture()
            if abs(t) <= qmax and bf16_bits_to_f64(bf16_bits(np.float32([t])))[0] == t]
    assert len(rows) >= 15 or bits == 4
    for e in (0, -3, 5):  # scale = 2^e, so x = t * 2^e and t = x * inv exactly
        G = 128
        x = np.zeros(G, np.float32)
        x[0] = qmax * 2.0 ** e
        for j, (t, _) in enumerate(rows):
            x[1 + j] = t * 2.0 ** e
        xb = bf16_bits(x)
        assert np.array_equal(bf16_bits_to_f64(xb), x.astype(np.float64))  # representable
        codes, scales = ref.act_quant(xb, G, bits)
        assert scales[0] == np.float32(2.0 ** e)
        got = codes_to_int(codes, bits)
        for j, (t, q) in enumerate(rows):
            assert got[1 + j] == q, (t, q, got[1 + j])


def test_ties_round_to_even_fp32_gradients(ref):
    rows = load_tie_fixture()
    G = 64
    g = np.zeros(G, np.float32)
    g[0] = -127.0 * 2.0 ** -20
    for j, (t, _) in enumerate(rows):
        g[1 + j] = t * 2.0 ** -20
    codes, scales = ref.grad_quant(g, G)
    assert scales[0] == np.float32(2.0 ** -20)
    assert codes[0] == -127
    for j, (t, q) in enumerate(rows):
        assert codes[1 + j] == q


# ---------------------------------------------------------------------------
# byte-level packing against a hand-written fixture
# ---------------------------------------------------------------------------

def test_nibble_packing_fixture(ref):
    # fixture: 16 values on a grid of step 1 with amax 7 -> codes = values;
    # expected bytes written by hand: low nibble = even element, two's complement
    vals, want_bytes = [], []
    with open(os.path.join(GOLDEN, "nibble_packing.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, rest = line.split(":")
            if key == "values":
                vals = [float(v) for v in rest.split()]
            elif key == "bytes":
                want_bytes = [int(b, 16) for b in rest.split()]
    xb = bf16_bits(np.array(vals, np.float32))
    codes, scales = ref.act_quant(xb, 16, 4)
    assert scales[0] == np.float32(1.0)
    assert list(codes) == want_bytes
    # and the same values as 8-bit codes are plain int8 in element order
    x8 = np.array(vals, np.float32) * np.float32(127.0 / 7.0)
    x8 = np.rint(x8)  # integers up to 127: exact in bf16
    c8, s8 = ref.act_quant(bf16_bits(x8), 16, 8)
    assert s8[0] == np.float32(1.0)
    assert np.array_equal(c8.view(np.int8).astype(np.float32), x8)


def load_plane_fixture(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, rest = line.split(":")
                out[key.strip()] = rest.split()
    return out


@pytest.mark.parametrize("bits,name", [(5, "plane_packing_5bit.txt"), (6, "plane_packing_6bit.txt")])
def test_plane_packing_fixtures(ref, bits, name):
    # two groups of 8 on a grid of step 1 (amax = qmax, so scale = 1 and code = value);
    # expected bytes written by hand: nibble plane first, plane of high bits after it
    fx = load_plane_fixture(name)
    vals = np.array([float(v) for v in fx["values"]], np.float32)
    want = [int(b, 16) for b in fx["nibble_plane"]] + [int(b, 16) for b in fx["high_plane"]]
    codes, scales = ref.act_quant(bf16_bits(vals), 8, bits)
    assert np.all(scales == 1.0)
    assert list(codes) == want
    y = ref.act_dequant(np.array(want, np.uint8), scales, vals.size, 8, bits)
    assert np.array_equal(bf16_bits_to_f64(y), vals.astype(np.float64))


def test_dequant_unpacks_what_quant_packed(ref):
    # decode side of the layout, including the code -8 / -128 that quant never emits
    codes = np.array([0x8F, 0x10, 0x7E, 0x98], np.uint8)   # elems: -1,-8, 0,1, -2,7, -8,-7
    scales = np.array([0.5], np.float32)
    y = ref.act_dequant(codes, scales, 8, 8, 4)
    want = np.array([-1, -8, 0, 1, -2, 7, -8, -7], np.float64) * 0.5
    assert np.array_equal(bf16_bits_to_f64(y), want)
    c8 = np.array([-128, 127, -1, 0, 5, -5, 64, -64], np.int8).view(np.uint8)
    y8 = ref.act_dequant(c8, np.array([2.0], np.float32), 8, 8, 8)
    assert np.array_equal(bf16_bits_to_f64(y8), c8.view(np.int8).astype(np.float64) * 2.0)


# ---------------------------------------------------------------------------
# closed forms and invariants
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("G", [64, 128])
def test_values_on_the_grid_are_reconstructed_exactly(ref, bits, G):
    qmax = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(11)
    n_groups = 64
    k = rng.integers(-qmax, qmax + 1, size=(n_groups, G))
    k[np.arange(n_groups), rng.integers(0, G, n_groups)] = qmax * rng.choice([-1, 1], n_groups)
    e = rng.integers(-40, 40, size=(n_groups, 1))
    x = (k * 2.0 ** e).astype(np.float32)
    xb = bf16_bits(x)
    assert np.array_equal(bf16_bits_to_f64(xb), x.astype(np.float64))
    codes, scales = ref.act_quant(xb, G, bits)
    assert np.array_equal(scales, (2.0 ** e[:, 0]).astype(np.float32))
    assert np.array_equal(codes_to_int(codes, bits).reshape(n_groups, G), k)
    y = ref.act_dequant(codes, scales, x.size, G, bits)
    assert np.array_equal(y, xb.reshape(-1))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_zero_groups(ref, bits):
    G = 128
    x = np.zeros((3, G), np.uint16)
    x[1] = bf16_bits(np.random.default_rng(0).standard_normal(G).astype(np.float32))
    x[2, 5] = 0x8000                      # a lone negative zero
    codes, scales = ref.act_quant(x, G, bits)
    assert scales[0] == 0.0 and scales[2] == 0.0 and scales[1] > 0.0
    q = codes_to_int(codes, bits).reshape(3, G)
    assert not q[0].any() and not q[2].any() and q[1].any()
    y = ref.act_dequant(codes, scales, 3 * G, G, bits).reshape(3, G)
    assert not y[0].any() and not y[2].any()   # +0.0 bit pattern


def test_tiny_amax_threshold(ref):
    G = 128
    below = np.float32(2.0 ** -101)
    at = np.float32(2.0 ** -100)
    g = np.zeros((2, G), np.float32)
    g[0, 3] = below
    g[0, 9] = -below
    g[1, 3] = at
    codes, scales = ref.grad_quant(g, G)
    assert scales[0] == 0.0 and not codes[:G].any()
    assert scales[1] == np.float32(2.0 ** -100) / np.float32(127.0)
    assert codes[G + 3] == 127


@pytest.mark.parametrize("bits", ALL_BITS)
def test_sign_symmetry(ref, bits):
    rng = np.random.default_rng(3)
    x = bf16_bits(rng.standard_normal(128 * 50).astype(np.float32) * 3.0)
    c1, s1 = ref.act_quant(x, 128, bits)
    c2, s2 = ref.act_quant(x ^ np.uint16(0x8000), 128, bits)
    assert np.array_equal(s1, s2)
    assert np.array_equal(codes_to_int(c1, bits), -codes_to_int(c2, bits))


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("G", [64, 128])
def test_round_trip_error_bound_and_extreme_code(ref, bits, G):
    qmax = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(17)
    x32 = rng.standard_t(3.0, size=(400, G)).astype(np.float32)
    x32[:, 7] *= 50.0
    x32 *= (10.0 ** rng.integers(-30, 30, size=(400, 1))).astype(np.float32)
    xb = bf16_bits(x32)
    xv = bf16_bits_to_f64(xb)
    codes, scales = ref.act_quant(xb, G, bits)
    q = codes_to_int(codes, bits).reshape(400, G)
    s = scales.astype(np.float64).reshape(400, 1)
    # scale = amax/qmax, correctly rounded: cross-check with numpy's IEEE float32 division
    amax = np.abs(xv).max(axis=1).astype(np.float32)
    assert np.array_equal(scales, amax / np.float32(qmax))
    # |x - q*scale| <= scale/2 in exact arithmetic.  In binary32 the code is taken from
    # t = RN(x * RN(qmax/amax)), off from x/scale by at most qmax * 2^-23, and the product
    # q * RN(amax/qmax) is off by at most qmax * 2^-23 scale units again, hence the bound
    # scale * (1/2 + qmax * 2^-22) (times 1 + 2^-20 for second-order terms).
    v32 = (q.astype(np.float32) * scales.reshape(400, 1))          # the fp32 product
    err = np.abs(xv - v32.astype(np.float64))
    assert np.all(err <= s * (0.5 + qmax * 2.0 ** -22) * (1.0 + 2.0 ** -20))
    # the slack only matters next to a rounding boundary; the bulk obeys scale/2 as such
    assert np.mean(err <= 0.5 * s) > 0.999
    # the abs-max element carries +-qmax, nothing lies beyond
    pos = np.abs(xv).argmax(axis=1)
    assert np.all(np.abs(q[np.arange(400), pos]) == qmax)
    assert np.abs(q).max() <= qmax


def test_gradient_quant_matches_numpy_float32_formulation(ref):
    # same reading written with numpy float32 array operations (IEEE, no fma)
    rng = np.random.default_rng(23)
    g = (rng.standard_normal((300, 128)) * 1e-4).astype(np.float32)
    g[rng.random(g.shape) < 0.001] *= 100.0
    codes, scales = ref.grad_quant(g, 128)
    amax = np.abs(g).max(axis=1)
    scale = amax / np.float32(127.0)
    inv = np.float32(127.0) / amax
    t = g * inv[:, None]
    assert t.dtype == np.float32
    want = np.clip(rint_half_even_f64(t.astype(np.float64)), -127, 127).astype(np.int8)
    assert np.array_equal(scales, scale)
    assert np.array_equal(codes.reshape(300, 128), want)
    # and the plain dequantization of those codes
    out = ref.grad_dequant(codes, scales, 128)
    assert np.array_equal(out.reshape(300, 128), want.astype(np.float32) * scale[:, None])


def test_inv_is_its_own_division_not_reciprocal_of_scale(ref):
    # find a group where RN(x * RN(qmax/amax)) and RN(x * RN(1/scale)) or RN(x/scale)
    # round differently, and check that the oracle follows the stated reading
    rng = np.random.default_rng(29)
    G, qmax = 128, 127
    found = 0
    for _ in range(4000):
        g = rng.standard_normal(G).astype(np.float32)
        amax = np.abs(g).max()
        scale = amax / np.float32(qmax)
        inv = np.float32(qmax) / amax
        alt1 = rint_half_even_f64((g * (np.float32(1.0) / scale)).astype(np.float64))
        alt2 = rint_half_even_f64((g / scale).astype(np.float64))
        want = rint_half_even_f64((g * inv).astype(np.float64))
        if np.array_equal(want, alt1) and np.array_equal(want, alt2):
            continue
        found += 1
        codes, _ = ref.grad_quant(g, G)
        assert np.array_equal(codes.astype(np.float64), np.clip(want, -qmax, qmax))
    assert found > 0


# ---------------------------------------------------------------------------
# dequantize: exact product, then bf16 round-to-nearest-even
# ---------------------------------------------------------------------------

def test_bf16_rounding_against_torch_and_rationals(ref):
    # a group of one 8-bit code equal to 1 turns act_dequant into bf16(scale)
    rng = np.random.default_rng(31)
    rand = rng.standard_normal(200000).astype(np.float32) * \
        (10.0 ** rng.integers(-37, 37, 200000)).astype(np.float32)
    # every bf16 value, every midpoint between neighbours (ties), and neighbours of midpoints
    b = all_finite_bf16_bits().astype(np.uint32) << 16
    ties = b | 0x8000
    vals = np.concatenate([b, ties, ties - 1, ties + 1, rand.view(np.uint32)]).astype(np.uint32)
    v = vals.view(np.float32)
    v = v[np.isfinite(v) & (np.abs(v) < 3.3e38)]
    y = ref.act_dequant(np.ones(v.size, np.uint8), v, v.size, 1, 8)
    want = torch.from_numpy(v.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y, want)
    for i in rng.integers(0, v.size, 300):           # and from first principles
        assert y[i] == bf16_rne_from_fraction(Fraction(float(v[i])))
    # scalar entry points agree
    assert ref.f32_to_bf16(1.00390625) == 0x3F80      # 1 + 2^-8: tie, even is 1.0
    assert ref.f32_to_bf16(1.01171875) == 0x3F82      # 1 + 3*2^-8: tie, even is 1+2^-6
    assert ref.bf16_to_f32(0x3F80) == 1.0 and ref.bf16_to_f32(0xC049) == -3.140625


@pytest.mark.parametrize("bits", ALL_BITS)
def test_dequant_every_code_times_scale_exact(ref, bits):
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    rng = np.random.default_rng(37)
    n_codes = hi - lo + 1
    G = n_codes
    assert G in (16, 32, 64, 256)
    scales = np.concatenate([
        rng.standard_normal(500).astype(np.float32) ** 2 *
        (10.0 ** rng.integers(-30, 30, 500)).astype(np.float32),
        np.array([1.0, 2.0 ** -107, 2.0 ** -126, 1e-42, 0.0, 2.0e36], np.float32)])
    scales = scales.astype(np.float32)
    q = np.tile(np.arange(lo, hi + 1, dtype=np.int32), (scales.size, 1))
    codes = pack_codes(q, bits)
    y = ref.act_dequant(codes, scales, q.size, G, bits).reshape(scales.size, G)
    prod = (q.astype(np.float64) * scales.astype(np.float64)[:, None]).astype(np.float32)
    want = torch.from_numpy(prod).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(y, want)


def test_codes_survive_requantization_on_power_of_two_scales(ref):
    rng = np.random.default_rng(41)
    G = 128
    k = rng.integers(-7, 8, size=(32, G))
    k[:, 0] = 7
    x = bf16_bits((k * 2.0 ** -4).astype(np.float32))
    c, s = ref.act_quant(x, G, 4)
    y = ref.act_dequant(c, s, x.size, G, 4)
    c2, s2 = ref.act_quant(y, G, 4)
    assert np.array_equal(c, c2) and np.array_equal(s, s2)


# ---------------------------------------------------------------------------
# argument checking and thread independence
# ---------------------------------------------------------------------------

def test_bad_arguments_are_rejected(ref):
    x = np.zeros(256, np.uint16)
    for group, bits in [(128, 3), (128, 16), (0, 4), (100, 4)]:
        with pytest.raises(ref.OracleError):
            ref.act_quant(x, group, bits)
    with pytest.raises(ref.OracleError):
        ref.grad_quant(np.zeros(100, np.float32), 64)


def test_result_does_not_depend_on_thread_count(ref):
    rng = np.random.default_rng(43)
    x = bf16_bits(rng.standard_normal(128 * 999).astype(np.float32))
    n = ref.max_threads()
    try:
        ref.set_threads(1)
        a = ref.act_quant(x, 128, 4)
        ref.set_threads(max(2, n))
        b = ref.act_quant(x, 128, 4)
    finally:
        ref.set_threads(n)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
