"""Pins of the oracle on non-finite inputs (CPU only).

Reading (the paper is silent): Inf and NaN propagate at group granularity.  A group that
holds one stores scale = quiet NaN (bits 0x7FC00000) and all-zero codes, so that all of it
reads back as NaN; the fp32 sums of the reduce and of the accumulation are treated the same
way, so a NaN scale in any chunk, or a sum that overflows binary32, gives a NaN group.

What fixes the expected values here, apart from the rule itself: groups are independent, so
every group without a non-finite value must come out exactly as it does when the poisoned
groups are replaced by zeros; a group of zeros has all-zero codes (pinned with the tiny-group
rule elsewhere), so the code bytes of the whole tensor must equal those of the zeroed tensor.
"""
import numpy as np
import pytest

QNAN = 0x7FC00000
POISONS_BF16 = {"+inf": 0x7F80, "-inf": 0xFF80, "nan": 0x7FC0, "nan_payload": 0x7FFF,
                "negative_nan": 0xFFC1, "signalling_nan": 0x7F81}
POISONS_F32 = {"+inf": 0x7F800000, "-inf": 0xFF800000, "nan": 0x7FC00000,
               "nan_low_payload": 0x7FC000FF, "all_ones": 0xFFFFFFFF, "signalling_nan": 0x7F800001}


def bf16_bits(a):
    """float32 array -> bf16 bit patterns by round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_is_nan(bits):
    bits = np.asarray(bits, np.uint16)
    return ((bits & 0x7F80) == 0x7F80) & ((bits & 0x007F) != 0)


def poisoned_activation(group, n_groups, poison_bits, where):
    rng = np.random.default_rng(1234)
    x = bf16_bits(rng.standard_normal(group * n_groups).astype(np.float32))
    clean = x.copy()
    for g, j in where:
        x[g * group + j] = poison_bits
        clean[g * group:(g + 1) * group] = 0
    return x, clean


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("poison", sorted(POISONS_BF16))
def test_activation_group_with_a_nonfinite_value(ref, bits, poison):
    group, n_groups = 128, 9
    where = [(0, 0), (3, 77), (8, 127)]                 # first, middle, last element of a group
    x, clean = poisoned_activation(group, n_groups, POISONS_BF16[poison], where)
    codes, scales = ref.act_quant(x, group, bits)
    want_codes, want_scales = ref.act_quant(clean, group, bits)
    bad = sorted({g for g, _ in where})
    good = [g for g in range(n_groups) if g not in bad]
    assert np.array_equal(codes, want_codes)            # poisoned groups: zero codes, like zeros
    assert np.all(scales.view(np.uint32)[bad] == QNAN)
    assert np.array_equal(scales.view(np.uint32)[good], want_scales.view(np.uint32)[good])
    assert np.all(want_scales[bad] == 0.0)              # (what the zeroed groups are compared with)
    y = ref.act_dequant(codes, scales, x.size, group, bits).reshape(n_groups, group)
    want_y = ref.act_dequant(want_codes, want_scales, x.size, group, bits).reshape(n_groups, group)
    assert bf16_is_nan(y[bad]).all()                    # the whole group, not only the element
    assert np.array_equal(y[good], want_y[good])
    assert not bf16_is_nan(y[good]).any()


@pytest.mark.parametrize("poison", sorted(POISONS_BF16))
def test_e2m1_activation_group_with_a_nonfinite_value(ref, poison):
    group, n_groups = 64, 6
    where = [(1, 5), (5, 63)]
    x, clean = poisoned_activation(group, n_groups, POISONS_BF16[poison], where)
    codes, scales = ref.fp4_act_quant(x, group)
    want_codes, want_scales = ref.fp4_act_quant(clean, group)
    bad = [1, 5]
    good = [0, 2, 3, 4]
    assert np.array_equal(codes, want_codes)
    assert np.all(codes.reshape(n_groups, -1)[bad] == 0)   # no sign bits left behind either
    assert np.all(scales.view(np.uint32)[bad] == QNAN)
    assert np.array_equal(scales.view(np.uint32)[good], want_scales.view(np.uint32)[good])
    y = ref.fp4_act_dequant(codes, scales, x.size, group).reshape(n_groups, group)
    assert bf16_is_nan(y[bad]).all() and not bf16_is_nan(y[good]).any()


def poisoned_gradient(group, n_groups, poison_bits, where):
    rng = np.random.default_rng(4321)
    g = (rng.standard_normal(group * n_groups) * 1e-3).astype(np.float32)
    clean = g.copy()
    for grp, j in where:
        g.view(np.uint32)[grp * group + j] = poison_bits
        clean[grp * group:(grp + 1) * group] = 0
    return g, clean


@pytest.mark.parametrize("poison", sorted(POISONS_F32))
@pytest.mark.parametrize("fp8", [False, True])
def test_gradient_group_with_a_nonfinite_value(ref, poison, fp8):
    group, n_groups = 128, 7
    where = [(2, 0), (6, 100)]
    g, clean = poisoned_gradient(group, n_groups, POISONS_F32[poison], where)
    quant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    dequant = ref.fp8_grad_dequant if fp8 else ref.grad_dequant
    codes, scales = quant(g, group)
    want_codes, want_scales = quant(clean, group)
    bad, good = [2, 6], [0, 1, 3, 4, 5]
    assert np.array_equal(codes, want_codes)
    assert np.all(codes.reshape(n_groups, group)[bad] == 0)
    assert np.all(scales.view(np.uint32)[bad] == QNAN)
    assert np.array_equal(scales.view(np.uint32)[good], want_scales.view(np.uint32)[good])
    out = dequant(codes, scales, group).reshape(n_groups, group)
    assert np.isnan(out[bad]).all() and np.isfinite(out[good]).all()


@pytest.mark.parametrize("fp8", [False, True])
def test_reduce_propagates_a_nan_scale_and_an_overflowing_sum(ref, fp8):
    group, n_groups, K = 64, 6, 3
    rng = np.random.default_rng(99)
    quant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    reduce_ = ref.fp8_grad_reduce_requant if fp8 else ref.grad_reduce_requant
    pairs = [quant((rng.standard_normal(group * n_groups) * 1e-2).astype(np.float32), group) for _ in range(K)]
    codes = np.stack([p[0] for p in pairs])
    scales = np.stack([p[1] for p in pairs])
    want_codes, want_scales = reduce_(codes, scales, group * n_groups, group)
    assert np.isfinite(want_scales).all()
    # group 1: chunk 2 arrives with a NaN scale (its sender saw a non-finite gradient);
    # group 4: two chunks whose full-scale terms are finite but whose sum is not:
    #          code of largest magnitude * 2^127 = 1.7e38..., twice that overflows binary32
    poisoned = scales.copy()
    poisoned.view(np.uint32)[2, 1] = QNAN
    poisoned[0, 4] = np.float32(2.0 ** 127) / (448.0 if fp8 else 127.0) * np.float32(1.5)
    poisoned[1, 4] = poisoned[0, 4]
    c2 = codes.copy()
    full = 0x7E if fp8 else 127                              # +448 in E4M3, +127 in int8
    c2[0, 4 * group] = full
    c2[1, 4 * group] = full
    got_codes, got_scales = reduce_(c2, poisoned, group * n_groups, group)
    bad, good = [1, 4], [0, 2, 3, 5]
    gc = got_codes.reshape(n_groups, group)
    assert np.all(gc[bad] == 0)
    assert np.all(got_scales.view(np.uint32)[bad] == QNAN)
    assert np.array_equal(gc[good], want_codes.reshape(n_groups, group)[good])
    assert np.array_equal(got_scales.view(np.uint32)[good], want_scales.view(np.uint32)[good])


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("addend", ["f32", "bf16"])
def test_accumulate_propagates(ref, fp8, addend):
    group, n_groups = 64, 5
    rng = np.random.default_rng(7)
    quant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    acc = ref.fp8_grad_accumulate if fp8 else ref.grad_accumulate
    main_c, main_s = quant((rng.standard_normal(group * n_groups) * 1e-2).astype(np.float32), group)
    g_new = (rng.standard_normal(group * n_groups) * 1e-2).astype(np.float32)
    g_in = bf16_bits(g_new) if addend == "bf16" else g_new
    want_c, want_s = acc(main_c, main_s, g_in, group)
    g_bad = g_in.copy()
    g_bad[0 * group + 3] = 0x7F80 if addend == "bf16" else np.float32(np.inf)     # Inf in the new gradient
    s_bad = main_s.copy()
    s_bad.view(np.uint32)[3] = QNAN                                               # stored group already NaN
    got_c, got_s = acc(main_c, s_bad, g_bad, group)
    bad, good = [0, 3], [1, 2, 4]
    assert np.all(got_c.reshape(n_groups, group)[bad] == 0)
    assert np.all(got_s.view(np.uint32)[bad] == QNAN)
    assert np.array_equal(got_c.reshape(n_groups, group)[good], want_c.reshape(n_groups, group)[good])
    assert np.array_equal(got_s.view(np.uint32)[good], want_s.view(np.uint32)[good])


def test_bf16_conversion_of_nonfinite_values(ref):
    inf = np.float32(np.inf)
    assert ref.f32_to_bf16(inf) == 0x7F80 and ref.f32_to_bf16(-inf) == 0xFF80
    # the largest finite binary32 is closer to 2^128 than to the largest bf16: it rounds to Inf
    assert ref.f32_to_bf16(np.float32(3.4028234663852886e38)) == 0x7F80
    for pattern in (0x7FC00000, 0x7F800001, 0x7FFFFFFF, 0xFFFFFFFF, 0xFFC00001, 0x7F80FFFF):
        f = np.array([pattern], np.uint32).view(np.float32)[0]
        assert bf16_is_nan(ref.f32_to_bf16(f)), hex(pattern)


def test_recompute_of_a_poisoned_group(ref):
    """RMSNorm of a row that holds a NaN group is NaN over the whole row (its mean square
    is); SiLU & Multiply is NaN exactly where either operand is; other rows are untouched."""
    group, rows, cols = 64, 4, 256
    rng = np.random.default_rng(5)
    x = bf16_bits(rng.standard_normal(rows * cols).astype(np.float32))
    codes, scales = ref.act_quant(x, group, 4)
    gamma = (1.0 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    want_y, want_r = ref.act_dequant_rmsnorm(codes, scales, rows, cols, group, 4, gamma, 1e-5)
    poisoned = scales.copy()
    poisoned.view(np.uint32)[2 * (cols // group) + 1] = QNAN        # row 2, second group
    y, r = ref.act_dequant_rmsnorm(codes, poisoned, rows, cols, group, 4, gamma, 1e-5)
    y, want_y = y.reshape(rows, cols), want_y.reshape(rows, cols)
    assert bf16_is_nan(y[2]).all() and np.isnan(r[2])
    assert np.array_equal(y[[0, 1, 3]], want_y[[0, 1, 3]])
    assert np.array_equal(r[[0, 1, 3]].view(np.uint32), want_r[[0, 1, 3]].view(np.uint32))
    u = bf16_bits(rng.standard_normal(rows * cols).astype(np.float32))
    ucodes, uscales = ref.act_quant(u, group, 8)
    want_z = ref.act_dequant_silu_mul(codes, scales, 4, ucodes, uscales, 8, rows * cols, group)
    z = ref.act_dequant_silu_mul(codes, poisoned, 4, ucodes, uscales, 8, rows * cols, group)
    lo = (2 * (cols // group) + 1) * group
    mask = np.zeros(rows * cols, bool)
    mask[lo:lo + group] = True
    assert bf16_is_nan(z[mask]).all()
    assert np.array_equal(z[~mask], want_z[~mask])
