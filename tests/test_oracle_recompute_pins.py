"""Pins for the oracle's fused dequantize + recompute functions (RMSNorm, SiLU & Multiply)."""
import numpy as np
import pytest
import torch

from exact import bf16_bits_to_f64, pack_codes


def bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_steps_apart(a_bits, b_bits):
    """Distance in bf16 steps between two arrays of bit patterns (sign-magnitude aware)."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(np.asarray(a_bits)) - key(np.asarray(b_bits)))


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_rmsnorm_matches_torch_on_the_dequantized_input(ref, bits):
    rng = np.random.default_rng(60 + bits)
    rows, cols, group = 37, 512, 128
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    x[:, 7] *= 30.0
    codes, scales = ref.act_quant(bf16_bits(x), group, bits)
    gamma = (1.0 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    y, r = ref.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, gamma, eps)
    # library cross-check in float64: torch's own rms_norm on the plain dequantized tensor
    xd = bf16_bits_to_f64(ref.act_dequant(codes, scales, rows * cols, group, bits)).reshape(rows, cols)
    t = torch.from_numpy(xd)
    want = torch.nn.functional.rms_norm(t, (cols,), torch.from_numpy(gamma.astype(np.float64)), eps).numpy()
    want_r = np.sqrt((xd ** 2).mean(axis=1) + eps)
    assert np.allclose(r, want_r, rtol=2e-7, atol=0)
    want_bits = bf16_bits(want.astype(np.float32))          # float64 -> float32 -> bf16
    d = bf16_steps_apart(y, want_bits.reshape(-1))
    assert d.max() <= 1 and np.mean(d == 0) > 0.999


def test_rmsnorm_closed_forms(ref):
    group, cols = 64, 256
    # a row of +-c: every x'^2 = c^2, r = sqrt(c^2 + eps), y = gamma * sign * c / r
    c = 0.5
    signs = np.where(np.arange(cols) % 3 == 0, -1.0, 1.0)
    x = (c * signs).astype(np.float32)[None, :]
    codes, scales = ref.act_quant(bf16_bits(x), group, 8)
    assert np.array_equal(bf16_bits_to_f64(ref.act_dequant(codes, scales, cols, group, 8)), x.reshape(-1))
    gamma = np.full(cols, 2.0, np.float32)
    for eps in (0.0, 0.75):
        y, r = ref.act_dequant_rmsnorm(codes, scales, 1, cols, group, 8, gamma, eps)
        assert r[0] == np.float32(np.sqrt(c * c + eps))
        want = bf16_bits((2.0 * signs * c / np.sqrt(c * c + eps)).astype(np.float32))
        assert np.array_equal(y, want)
    # a zero row: r = sqrt(eps), y = 0
    z_codes = np.zeros(cols, np.uint8)
    y, r = ref.act_dequant_rmsnorm(z_codes, np.zeros(cols // group, np.float32), 1, cols, group, 8, gamma, 1e-6)
    assert r[0] == np.float32(1e-3) and not y.any()
    # scale invariance: multiplying the scales by 4 (exact) multiplies r by 4 and leaves y alone when eps = 0
    rng = np.random.default_rng(3)
    q = rng.integers(-127, 128, size=2 * cols)
    codes = pack_codes(q, 8)
    s1 = (rng.random(2 * cols // group) + 0.5).astype(np.float32)
    y1, r1 = ref.act_dequant_rmsnorm(codes, s1, 2, cols, group, 8, gamma, 0.0)
    y4, r4 = ref.act_dequant_rmsnorm(codes, s1 * 4, 2, cols, group, 8, gamma, 0.0)
    assert np.array_equal(y1, y4) and np.allclose(r4, 4 * r1, rtol=1e-7)
    # rows are independent
    y_row1, r_row1 = ref.act_dequant_rmsnorm(codes[cols:], s1[cols // group:], 1, cols, group, 8, gamma, 0.0)
    assert np.array_equal(y_row1, y1[cols:]) and r_row1[0] == r1[1]


@pytest.mark.parametrize("gate_bits,up_bits", [(4, 4), (8, 4), (5, 6), (8, 8)])
def test_silu_mul_matches_torch_on_the_dequantized_inputs(ref, gate_bits, up_bits):
    rng = np.random.default_rng(70 + gate_bits + up_bits)
    n, group = 128 * 300, 128
    g = (rng.standard_normal(n) * 3).astype(np.float32)
    u = rng.standard_normal(n).astype(np.float32)
    gc, gs = ref.act_quant(bf16_bits(g), group, gate_bits)
    uc, us = ref.act_quant(bf16_bits(u), group, up_bits)
    z = ref.act_dequant_silu_mul(gc, gs, gate_bits, uc, us, up_bits, n, group)
    gd = torch.from_numpy(bf16_bits_to_f64(ref.act_dequant(gc, gs, n, group, gate_bits)))
    ud = torch.from_numpy(bf16_bits_to_f64(ref.act_dequant(uc, us, n, group, up_bits)))
    want = (torch.nn.functional.silu(gd) * ud).numpy()
    d = bf16_steps_apart(z, bf16_bits(want.astype(np.float32)))
    assert d.max() <= 1 and np.mean(d == 0) > 0.999


def test_silu_mul_closed_forms(ref):
    group = 64
    # gate = 0 -> z = 0; large positive gate -> z = u * g; large negative gate -> z -> 0
    q = np.zeros(group, np.int64)
    q[:4] = [0, 127, -127, 64]
    gc = pack_codes(q, 8)
    gs = np.array([0.5], np.float32)                 # gate values 0, 63.5, -63.5, 32
    uq = np.full(group, 4, np.int64)
    uc = pack_codes(uq, 8)
    us = np.array([0.25], np.float32)                # up = 1.0 everywhere
    z = bf16_bits_to_f64(ref.act_dequant_silu_mul(gc, gs, 8, uc, us, 8, group, group))
    assert z[0] == 0.0
    assert z[1] == 63.5 and z[3] == 32.0             # sigma = 1 to within bf16
    assert abs(z[2]) < 1e-20                         # -63.5 * exp(-63.5)
    # symmetry: silu(g) - silu(-g) = g, with u = 1
    q2 = np.zeros(group, np.int64)
    q2[:6] = [3, -3, 40, -40, 101, -101]
    z2 = bf16_bits_to_f64(ref.act_dequant_silu_mul(pack_codes(q2, 8), np.array([2.0 ** -5], np.float32), 8,
                                                  uc, us, 8, group, group))
    for k in range(0, 6, 2):
        g = q2[k] * 2.0 ** -5
        assert abs((z2[k] - z2[k + 1]) - g) <= abs(g) * 2.0 ** -7


# ---- the forward side: plain layer definitions on the original inputs -----------------

def test_rmsnorm_forward_matches_torch(ref):
    rng = np.random.default_rng(90)
    rows, cols = 29, 640
    xb = bf16_bits((rng.standard_normal((rows, cols)) * 2).astype(np.float32))
    gamma = (1.0 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    y, r = ref.rmsnorm_fwd(xb, rows, cols, gamma, 1e-5)
    xd = torch.from_numpy(bf16_bits_to_f64(xb).reshape(rows, cols))
    want = torch.nn.functional.rms_norm(xd, (cols,), torch.from_numpy(gamma.astype(np.float64)), 1e-5).numpy()
    assert np.allclose(r, np.sqrt((xd.numpy() ** 2).mean(axis=1) + 1e-5), rtol=2e-7)
    d = bf16_steps_apart(y, bf16_bits(want.astype(np.float32)).reshape(-1))
    assert d.max() <= 1 and np.mean(d == 0) > 0.999
    # closed form: a row of +-c
    row = bf16_bits(np.where(np.arange(cols) % 2 == 0, 0.25, -0.25).astype(np.float32))
    y1, r1 = ref.rmsnorm_fwd(row, 1, cols, np.full(cols, 3.0, np.float32), 0.0)
    assert r1[0] == 0.25 and np.array_equal(bf16_bits_to_f64(y1), np.where(np.arange(cols) % 2 == 0, 3.0, -3.0))


def test_silu_mul_forward_matches_torch(ref):
    rng = np.random.default_rng(91)
    n = 5000
    gb = bf16_bits((rng.standard_normal(n) * 4).astype(np.float32))
    ub = bf16_bits(rng.standard_normal(n).astype(np.float32))
    z = ref.silu_mul_fwd(gb, ub)
    g = torch.from_numpy(bf16_bits_to_f64(gb))
    u = torch.from_numpy(bf16_bits_to_f64(ub))
    want = (torch.nn.functional.silu(g) * u).numpy()
    d = bf16_steps_apart(z, bf16_bits(want.astype(np.float32)))
    assert d.max() <= 1 and np.mean(d == 0) > 0.999
    zero = ref.silu_mul_fwd(np.zeros(8, np.uint16), ub[:8])
    assert not (zero & 0x7FFF).any()
