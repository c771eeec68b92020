"""Pins for the oracle's local reduce + requantize, local accumulation and DBCA helper."""
from fractions import Fraction
import os

import numpy as np
import pytest

from exact import f32_fraction, fraction_to_f32, rint_half_even_f64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def exact_fma_chain(codes, scales, group):
    """acc_i = fma(...fma(fma(0, .), .)) with ONE rounding per step, from rationals."""
    K, n = codes.shape
    out = np.zeros(n, np.float32)
    for i in range(n):
        acc = Fraction(0)
        for k in range(K):
            exact = Fraction(int(codes[k, i])) * f32_fraction(scales[k, i // group]) + acc
            acc = Fraction(float(fraction_to_f32(exact)))
        out[i] = np.float32(float(acc))
    return out


def quant8_numpy(acc, group):
    """The 8-bit group quantizer written with numpy float32 array operations."""
    a = acc.reshape(-1, group)
    amax = np.abs(a).max(axis=1)
    live = amax >= np.float32(2.0 ** -100)
    safe = np.where(live, amax, np.float32(1.0))
    scale = np.where(live, safe / np.float32(127.0), np.float32(0.0)).astype(np.float32)
    inv = np.float32(127.0) / safe
    t = a * inv[:, None]
    q = np.clip(rint_half_even_f64(t.astype(np.float64)), -127, 127)
    q = np.where(live[:, None], q, 0.0).astype(np.int8)
    return q.reshape(-1), scale


def random_chunks(rng, K, n, group, stride_pad=0):
    codes = rng.integers(-127, 128, size=(K, n + stride_pad)).astype(np.int8)
    scales = (rng.random((K, n // group + (1 if stride_pad else 0))) * 1e-5 + 1e-7).astype(np.float32)
    return codes, scales


@pytest.mark.parametrize("K,group,n_groups", [(1, 8, 3), (3, 8, 4), (4, 16, 2), (8, 64, 2), (16, 128, 1)])
def test_reduce_matches_exact_fma_chain(ref, K, group, n_groups):
    rng = np.random.default_rng(100 + K)
    n = group * n_groups
    codes, scales = random_chunks(rng, K, n, group, stride_pad=group)  # strides > extents
    acc = exact_fma_chain(codes[:, :n], scales, group)
    want_codes, want_scales = quant8_numpy(acc, group)
    got_codes, got_scales = ref.grad_reduce_requant(codes, scales, n, group)
    assert np.array_equal(got_scales.view(np.uint32), want_scales.view(np.uint32))
    assert np.array_equal(got_codes, want_codes)


def test_summation_order_is_chunk_order(ref):
    # three terms whose fp32 sum depends on the order: (big + -big) + small  vs  big + (-big + small)
    group = 8
    codes = np.zeros((3, group), np.int8)
    scales = np.zeros((3, 1), np.float32)
    codes[0, :] = 127; scales[0, 0] = 1.0            # 127
    codes[1, :] = -127; scales[1, 0] = 1.0           # -127
    codes[2, :] = 1; scales[2, 0] = 2.0 ** -30       # tiny: absorbed if added to 127 first
    codes[:, 0] = [100, 0, 0]                        # keeps the group's amax away from the tiny sum
    c012, s012 = ref.grad_reduce_requant(codes, scales, group, group)
    perm = [0, 2, 1]
    c021, s021 = ref.grad_reduce_requant(codes[perm], scales[perm], group, group)
    # order 0,1,2: elements 1.. sum to exactly 2^-30; order 0,2,1: the tiny term is lost -> 0
    assert s012[0] == np.float32(100.0) / np.float32(127.0)
    assert c012[0] == 127 and c021[0] == 127
    acc012 = exact_fma_chain(codes, scales, group)
    acc021 = exact_fma_chain(codes[perm], scales[perm], group)
    assert acc012[1] == np.float32(2.0 ** -30) and acc021[1] == 0.0
    assert np.array_equal(c012, quant8_numpy(acc012, group)[0])
    assert np.array_equal(c021, quant8_numpy(acc021, group)[0])


def test_fused_multiply_add_not_two_roundings(ref):
    # c*s + acc where rounding the product first would change the result
    group = 8
    found = 0
    rng = np.random.default_rng(7)
    for _ in range(2000):
        codes = rng.integers(-127, 128, size=(2, group)).astype(np.int8)
        scales = (rng.random((2, 1)) + 0.5).astype(np.float32)
        fused = exact_fma_chain(codes, scales, group)
        p0 = codes[0].astype(np.float32) * scales[0, 0]
        p1 = codes[1].astype(np.float32) * scales[1, 0]
        unfused = (p0 + p1).astype(np.float32)
        if np.array_equal(fused, unfused):
            continue
        want = quant8_numpy(fused, group)
        other = quant8_numpy(unfused, group)
        if np.array_equal(want[0], other[0]) and np.array_equal(want[1], other[1]):
            continue
        found += 1
        got = ref.grad_reduce_requant(codes, scales, group, group)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
    assert found > 0


@pytest.mark.parametrize("K", [1, 2, 4, 8, 16, 64])
def test_identical_chunks_power_of_two_scale(ref, K):
    # K copies of (q, 2^e): acc = K*q*2^e exactly; requantized scale = K*2^e*max|q|/127
    group, e = 128, -12
    rng = np.random.default_rng(K)
    q = rng.integers(-127, 128, size=group * 4).astype(np.int8)
    q[::group] = 127
    codes = np.tile(q, (K, 1))
    scales = np.full((K, 4), 2.0 ** e, np.float32)
    out_c, out_s = ref.grad_reduce_requant(codes, scales, q.size, group)
    if K & (K - 1) == 0:
        assert np.all(out_s == np.float32(K * 2.0 ** e))
        assert np.array_equal(out_c, q)          # same codes, scale multiplied by K
    else:
        assert np.allclose(out_s, K * 2.0 ** e, rtol=1e-6)


def test_cancelling_chunks_give_a_zero_group(ref):
    group = 64
    rng = np.random.default_rng(9)
    q = rng.integers(-127, 128, size=group * 2).astype(np.int8)
    codes = np.stack([q, -q, q, -q])
    scales = np.full((4, 2), 0.375, np.float32)       # few significant bits: q * s is exact
    scales[2:, :] = 1.25 * 2.0 ** -10
    out_c, out_s = ref.grad_reduce_requant(codes, scales, q.size, group)
    assert not out_c.any() and not out_s.any()
    # with a scale whose products are inexact, the fused multiply-add leaves the rounding
    # residual RN(q*s) - q*s behind instead of zero: a signature of the single rounding
    scales[:2, :] = np.float32(0.37)
    out_c, out_s = ref.grad_reduce_requant(codes[:2], scales[:2], q.size, group)
    resid = np.array([float(Fraction(float(np.float32(int(v)) * np.float32(0.37)))
                            - Fraction(int(v)) * f32_fraction(np.float32(0.37))) for v in q])
    want = quant8_numpy(resid.astype(np.float32), group)
    assert resid.any()
    assert np.array_equal(out_c, want[0]) and np.array_equal(out_s, want[1])


def test_reduce_never_saturates_and_tracks_the_exact_sum(ref):
    # the paper's point: summing in fp32 and requantizing cannot overflow; the largest
    # output code is exactly +-127 in every live group, and the fp32 sum stays within
    # K rounding errors of the binary64 sum
    group, K, n = 128, 16, 128 * 200
    rng = np.random.default_rng(13)
    g = [(rng.standard_normal(n) * 1e-4).astype(np.float32) for _ in range(K)]
    pairs = [ref.grad_quant(x, group) for x in g]
    codes = np.stack([p[0] for p in pairs])
    scales = np.stack([p[1] for p in pairs])
    out_c, out_s = ref.grad_reduce_requant(codes, scales, n, group)
    assert np.all(np.abs(out_c.reshape(-1, group).astype(np.int32)).max(axis=1) == 127)
    s64, a64 = ref.grad_reduce_f64(codes, scales, n, group)
    # independent check of the f64 sum itself
    want64 = (codes.astype(np.float64) * np.repeat(scales.astype(np.float64), group, axis=1)).sum(axis=0)
    assert np.allclose(s64, want64, rtol=1e-12, atol=1e-18)
    deq = out_c.astype(np.float64) * np.repeat(out_s.astype(np.float64), group)
    step = np.repeat(out_s.astype(np.float64), group)
    assert np.all(np.abs(deq - s64) <= 0.5 * step * (1 + 2.0 ** -14) + K * 2.0 ** -24 * a64)
    # the requantized sum approximates the sum of the ORIGINAL fp32 gradients too
    true = np.sum(np.stack(g).astype(np.float64), axis=0)
    in_step = np.repeat(scales.astype(np.float64), group, axis=1).sum(axis=0)
    assert np.all(np.abs(deq - true) <= 0.5 * in_step * 1.001 + 0.5 * step * 1.001)


def test_k1_power_of_two_scale_is_identity(ref):
    group = 128
    rng = np.random.default_rng(21)
    q = rng.integers(-127, 128, size=group * 8).astype(np.int8)
    q[5::group] = -127
    scales = (2.0 ** rng.integers(-30, 5, size=8)).astype(np.float32)
    out_c, out_s = ref.grad_reduce_requant(q[None, :], scales[None, :], q.size, group)
    assert np.array_equal(out_c, q) and np.array_equal(out_s, scales)


def test_reduce_rejects_bad_arguments(ref):
    codes = np.zeros((2, 128), np.int8)
    scales = np.zeros((2, 1), np.float32)
    with pytest.raises(ref.OracleError):
        ref.grad_reduce_requant(codes, scales, 256, 128)       # stride < numel
    with pytest.raises(ref.OracleError):
        ref.grad_reduce_requant(np.zeros((65, 128), np.int8), np.zeros((65, 1), np.float32), 128, 128)


# ---- local accumulation into the stored 8-bit gradient ----------------------

@pytest.mark.parametrize("as_bf16", [False, True])
def test_accumulate_matches_exact_arithmetic(ref, as_bf16):
    import torch
    group, n = 16, 64
    rng = np.random.default_rng(55)
    main_c = rng.integers(-127, 128, size=n).astype(np.int8)
    main_s = (rng.random(n // group) * 1e-3).astype(np.float32)
    g32 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    if as_bf16:
        t = torch.from_numpy(g32).to(torch.bfloat16)
        g_in = t.view(torch.int16).numpy().view(np.uint16)
        g32 = t.to(torch.float32).numpy()
    else:
        g_in = g32
    acc = np.zeros(n, np.float32)
    for i in range(n):
        acc[i] = fraction_to_f32(Fraction(int(main_c[i])) * f32_fraction(main_s[i // group])
                                 + f32_fraction(g32[i]))
    want = quant8_numpy(acc, group)
    got = ref.grad_accumulate(main_c, main_s, g_in, group)
    assert np.array_equal(got[0], want[0])
    assert np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))


def test_accumulate_onto_zero_main_gradient_equals_grad_quant(ref):
    group, n = 128, 128 * 40
    rng = np.random.default_rng(56)
    g = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    a = ref.grad_accumulate(np.zeros(n, np.int8), np.zeros(n // group, np.float32), g, group)
    b = ref.grad_quant(g, group)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ---- Dynamic Bit-width Compensation: the values the paper prints ------------

def load_kv(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split(":")
                out[k.strip()] = v.split()
    return out


def test_dbca_four_stage_values_from_the_paper(ref):
    gold = load_kv("dbca_four_stages.txt")
    n = int(gold["n_stages"][0])
    stored = [ref.dbca_stored_microbatches(n, i) for i in range(1, n + 1)]
    bits = [ref.dbca_bits(n, i) for i in range(1, n + 1)]
    assert stored == [int(v) for v in gold["stored_microbatches"]]
    assert bits == [int(v) for v in gold["bits"]]
    assert stored[0] / stored[-1] == pytest.approx(float(gold["ratio_first_to_last"][0]))


def test_dbca_general_properties(ref):
    for n in range(1, 17):
        stored = [ref.dbca_stored_microbatches(n, i) for i in range(1, n + 1)]
        bits = [ref.dbca_bits(n, i) for i in range(1, n + 1)]
        assert stored[-1] == n + 1                      # last stage: n + 1 micro-batches
        assert all(a - b == 2 for a, b in zip(stored, stored[1:]))
        assert bits[0] == 4                             # first stage keeps the minimum
        assert bits == sorted(bits) and all(4 <= b <= 8 for b in bits)
        # memory never exceeds the first stage's: bits_i * N_i <= 4 * N_1 unless rounded up
        for b, s in zip(bits, stored):
            assert (b - 0.5) * s <= 4 * stored[0] or b == 4
    with pytest.raises(ref.OracleError):
        ref.dbca_bits(4, 5)
    with pytest.raises(ref.OracleError):
        ref.dbca_bits(0, 1)
