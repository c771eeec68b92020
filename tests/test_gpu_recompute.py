"""GPU parity for dequantize fused with the Case-1 recompute (RMSNorm, SiLU & Multiply).

The oracle is the plain binary64 definition; the kernels compute in binary32, whose result
before the final rounding is within ~1e-5 relative of the exact one (cols * 2^-24 for the sum
of squares at worst, a few 1e-6 for exp), far below bf16's half step of 2^-9.  Bar: the bf16
outputs are equal, or one bf16 step apart where the exact
value sits within ~1e-5 relative of a rounding boundary (at most 0.5 % of the elements);
values whose exact magnitude is below 2^-100 (SiLU of a gate below about -70) only need to
come out below 2^-100 as well; r agrees to 2e-6 relative.
"""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def agoq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_00539_amd as lib
    lib.load_library()
    return lib


def steps_apart(a_bits, b_bits):
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(np.asarray(a_bits)) - key(np.asarray(b_bits)))


def bits_of(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)


TINY = 2.0 ** -100     # the method's own "this is zero" threshold; below it only smallness is compared


def bf16_value(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_close_bf16(got_bits, want_bits):
    d = steps_apart(got_bits, want_bits)
    both_tiny = (np.abs(bf16_value(got_bits)) < TINY) & (np.abs(bf16_value(want_bits)) < TINY)
    d = np.where(both_tiny, 0, d)
    assert d.max() <= 1, "more than one bf16 step apart"
    assert np.mean(d == 0) >= 0.995, "too many elements off by one step: %.4f" % np.mean(d != 0)


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("rows,cols", [(3, 128), (17, 1024), (64, 4096), (33, 5120), (5, 14336), (2, 16384), (7, 2048 + 128)])
def test_dequant_rmsnorm(agoq, ref, rows, cols, group, bits):
    x = wl.act_host(rows, cols, 7000 + rows + cols, "student_t3", max(1, cols // 100), 50.0)
    codes, scales = ref.act_quant(x, group, bits)
    rng = np.random.default_rng(cols)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    want_y, want_r = ref.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, gamma, eps)
    y, r = agoq.act_dequant_rmsnorm(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                                    rows, cols, group, bits, torch.from_numpy(gamma).cuda(), eps)
    torch.cuda.synchronize()
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)


def test_dequant_rmsnorm_zero_rows_and_eps(agoq, ref):
    rows, cols, group, bits = 4, 512, 128, 4
    x = wl.act_host(rows, cols, 1)
    x[1] = 0
    x[3] = 0x8000
    codes, scales = ref.act_quant(x, group, bits)
    gamma = np.ones(cols, np.float32)
    for eps in (1e-6, 0.25):
        want_y, want_r = ref.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, gamma, eps)
        y, r = agoq.act_dequant_rmsnorm(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                                        rows, cols, group, bits, torch.from_numpy(gamma).cuda(), eps)
        torch.cuda.synchronize()
        assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6)
        assert abs(float(r.cpu().numpy()[1]) - np.sqrt(eps)) <= 2e-6 * np.sqrt(eps)
        check_close_bf16(bits_of(y), want_y)
        assert not bits_of(y).reshape(rows, cols)[1].any()


@pytest.mark.parametrize("gate_bits,up_bits", [(4, 4), (8, 4), (4, 8), (5, 5), (6, 6), (5, 8), (8, 8)])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 9, 2 * 512 * 2 * 8 // 64 + 5, 30011])
def test_dequant_silu_mul(agoq, ref, n_groups, group, gate_bits, up_bits):
    n = n_groups * group
    rng = np.random.default_rng(8000 + n_groups)
    g = (rng.standard_normal(n) * 4).astype(np.float32)
    g[::1000] *= 30.0                                     # |gate| up to ~100: exp(-g) overflows in fp32
    u = rng.standard_normal(n).astype(np.float32)
    gb = torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ub = torch.from_numpy(u).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    gc, gs = ref.act_quant(gb, group, gate_bits)
    uc, us = ref.act_quant(ub, group, up_bits)
    want = ref.act_dequant_silu_mul(gc, gs, gate_bits, uc, us, up_bits, n, group)
    z = agoq.act_dequant_silu_mul(torch.from_numpy(gc).cuda(), torch.from_numpy(gs).cuda(), gate_bits,
                                  torch.from_numpy(uc).cuda(), torch.from_numpy(us).cuda(), up_bits, n, group)
    torch.cuda.synchronize()
    got = bits_of(z)
    assert not np.any((got & 0x7F80) == 0x7F80), "NaN or Inf in the output"
    check_close_bf16(got, want)


def test_recompute_error_codes(agoq):
    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    c = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    s = torch.zeros(64, dtype=torch.float32, device="cuda")
    gm = torch.ones(1024, dtype=torch.float32, device="cuda")
    y = torch.zeros(8192, dtype=torch.bfloat16, device="cuda")
    r = torch.zeros(8, dtype=torch.float32, device="cuda")
    pc, ps, pg, py, pr = (P(t.data_ptr()) for t in (c, s, gm, y, r))
    f = ctypes.c_float(1e-5)
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 1024, 128, 4, None, f, py, pr, None) == 1
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 1024, 128, 7, pg, f, py, pr, None) == 2
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 1024, 32, 4, pg, f, py, pr, None) == 3
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 1000, 128, 4, pg, f, py, pr, None) == 4
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 16384 + 128, 128, 4, pg, f, py, pr, None) == 4
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 0, 1024, 128, 4, pg, f, py, pr, None) == 4
    assert L.agoq_act_dequant_rmsnorm(pc, ps, 8, 1024, 128, 4, P(gm.data_ptr() + 4), f, py, pr, None) == 5
    assert L.agoq_act_dequant_silu_mul(pc, ps, 4, None, ps, 4, 1024, 128, py, None) == 1
    assert L.agoq_act_dequant_silu_mul(pc, ps, 3, pc, ps, 4, 1024, 128, py, None) == 2
    assert L.agoq_act_dequant_silu_mul(pc, ps, 4, pc, ps, 9, 1024, 128, py, None) == 2
    assert L.agoq_act_dequant_silu_mul(pc, ps, 4, pc, ps, 4, 1024, 100, py, None) == 3
    assert L.agoq_act_dequant_silu_mul(pc, ps, 4, pc, ps, 4, 1000, 128, py, None) == 4
    torch.cuda.synchronize()
    assert not bool(y.view(torch.int16).any())


# ---- forward side: compute the layer and store its quantized input in one pass ---------

def dev_bf16(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda().view(torch.bfloat16)


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("rows,cols", [(3, 128), (17, 1024), (64, 4096), (33, 5120), (5, 14336), (2, 16384)])
def test_rmsnorm_forward_with_quantized_input(agoq, ref, rows, cols, group, bits):
    x = wl.act_host(rows, cols, 9000 + rows + cols, "student_t3", max(1, cols // 100), 50.0)
    if rows > 4:
        x[2] = 0                                                   # a zero row: dead groups, r = sqrt(eps)
    rng = np.random.default_rng(cols + 1)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x), torch.from_numpy(gamma).cuda(), eps, group, bits)
    torch.cuda.synchronize()
    wc, ws = ref.act_quant(x, group, bits)                          # the stored form: bit for bit
    assert np.array_equal(codes.cpu().numpy(), wc)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    want_y, want_r = ref.rmsnorm_fwd(x, rows, cols, gamma, eps)      # the layer output: binary64 definition
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)


@pytest.mark.parametrize("gate_bits,up_bits", [(4, 4), (8, 4), (5, 6), (6, 5), (8, 8)])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 9, 2 * 128 * 2 * 8 // 64 + 5, 30011])
def test_silu_mul_forward_with_quantized_inputs(agoq, ref, n_groups, group, gate_bits, up_bits):
    n = n_groups * group
    rng = np.random.default_rng(9500 + n_groups)
    g = (rng.standard_normal(n) * 4).astype(np.float32)
    g[::1000] *= 30.0
    u = rng.standard_normal(n).astype(np.float32)
    if n_groups > 4:
        g[group: 2 * group] = 0.0
        u[2 * group: 3 * group] = -0.0
    gb = torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ub = torch.from_numpy(u).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    z, gc, gs, uc, us = agoq.silu_mul_fwd_quant(dev_bf16(gb), dev_bf16(ub), group, gate_bits, up_bits)
    torch.cuda.synchronize()
    for got_c, got_s, bits, src in ((gc, gs, gate_bits, gb), (uc, us, up_bits, ub)):
        wc, ws = ref.act_quant(src, group, bits)
        assert np.array_equal(got_c.cpu().numpy(), wc)
        assert np.array_equal(got_s.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    got = bits_of(z)
    assert not np.any((got & 0x7F80) == 0x7F80), "NaN or Inf in the output"
    check_close_bf16(got, ref.silu_mul_fwd(gb, ub))


def test_forward_then_backward_round_trip(agoq, ref):
    # what the backward recompute returns is the forward output of the dequantized input
    rows, cols, group, bits = 48, 4096, 128, 4
    x = wl.act_host(rows, cols, 77, "normal", 20, 30.0)
    gamma = np.ones(cols, np.float32)
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x), torch.from_numpy(gamma).cuda(), 1e-5, group, bits)
    y2, r2 = agoq.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, torch.from_numpy(gamma).cuda(), 1e-5)
    torch.cuda.synchronize()
    xd = ref.act_dequant(*ref.act_quant(x, group, bits), rows * cols, group, bits)
    want_y2, want_r2 = ref.rmsnorm_fwd(xd, rows, cols, gamma, 1e-5)
    assert np.allclose(r2.cpu().numpy(), want_r2, rtol=2e-6)
    check_close_bf16(bits_of(y2), want_y2)
    # 4-bit storage perturbs the normalized output by a bounded amount (step/2 per element / r)
    a = y.float().cpu().numpy()
    b = y2.float().cpu().numpy()
    assert np.abs(a - b).max() < 0.5 * 30 * 6 / 7          # outlier channel: amax ~ 30 * 5 sigma over qmax
    assert np.median(np.abs(a - b)) < 0.3


def test_forward_fused_error_codes(agoq):
    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    x = torch.zeros(8 * 1024, dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(8 * 1024, dtype=torch.bfloat16, device="cuda")
    gm = torch.ones(1024, dtype=torch.float32, device="cuda")
    c = torch.zeros(8 * 1024, dtype=torch.uint8, device="cuda")
    s = torch.zeros(128, dtype=torch.float32, device="cuda")
    px, py, pg, pc, ps = (P(t.data_ptr()) for t in (x, y, gm, c, s))
    f = ctypes.c_float(1e-5)
    assert L.agoq_rmsnorm_fwd_quant(None, 8, 1024, pg, f, 128, 4, py, None, pc, ps, None) == 1
    assert L.agoq_rmsnorm_fwd_quant(px, 8, 1024, pg, f, 128, 7, py, None, pc, ps, None) == 2
    assert L.agoq_rmsnorm_fwd_quant(px, 8, 1024, pg, f, 96, 4, py, None, pc, ps, None) == 3
    assert L.agoq_rmsnorm_fwd_quant(px, 8, 1000, pg, f, 128, 4, py, None, pc, ps, None) == 4
    assert L.agoq_rmsnorm_fwd_quant(px, 8, 1024, pg, f, 128, 4, P(y.data_ptr() + 2), None, pc, ps, None) == 5
    assert L.agoq_silu_mul_fwd_quant(px, None, 1024, 128, 4, 4, py, pc, ps, pc, ps, None) == 1
    assert L.agoq_silu_mul_fwd_quant(px, px, 1024, 128, 4, 9, py, pc, ps, pc, ps, None) == 2
    assert L.agoq_silu_mul_fwd_quant(px, px, 1000, 128, 4, 4, py, pc, ps, pc, ps, None) == 4
    torch.cuda.synchronize()
    assert not bool(y.view(torch.int16).any()) and not bool(c.any())


# ---- the same four calls on E2M1 codes --------------------------------------------------
# Oracle: the E2M1 dequantize of the oracle gives x' (bf16), and the layer's binary64
# definition is applied to x'; the stored form must equal the oracle's E2M1 quantize bit for bit.

@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("rows,cols", [(3, 128), (17, 1024), (64, 4096), (33, 5120), (5, 14336), (2, 16384)])
def test_fp4_dequant_rmsnorm(agoq, ref, rows, cols, group):
    x = wl.act_host(rows, cols, 11000 + rows + cols, "student_t3", max(1, cols // 100), 50.0)
    if rows > 4:
        x[1] = 0
    codes, scales = ref.fp4_act_quant(x, group)
    xd = ref.fp4_act_dequant(codes, scales, rows * cols, group)
    rng = np.random.default_rng(cols + 3)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    want_y, want_r = ref.rmsnorm_fwd(xd, rows, cols, gamma, eps)
    y, r = agoq.act_dequant_rmsnorm(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                                    rows, cols, group, 4, torch.from_numpy(gamma).cuda(), eps, fp4=True)
    torch.cuda.synchronize()
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 9, 133, 30011])
def test_fp4_dequant_silu_mul_and_forward(agoq, ref, n_groups, group):
    n = n_groups * group
    rng = np.random.default_rng(11500 + n_groups)
    g = (rng.standard_normal(n) * 4).astype(np.float32)
    g[::1000] *= 30.0
    u = rng.standard_normal(n).astype(np.float32)
    if n_groups > 4:
        g[group: 2 * group] = 0.0
        u[2 * group: 3 * group] = -0.0
    gb = torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ub = torch.from_numpy(u).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # forward: z from the exact inputs, stored form = the oracle's E2M1 quantize
    z, gc, gs, uc, us = agoq.silu_mul_fwd_quant(dev_bf16(gb), dev_bf16(ub), group, 4, 4, fp4=True)
    torch.cuda.synchronize()
    stored = []
    for got_c, got_s, src in ((gc, gs, gb), (uc, us, ub)):
        wc, ws = ref.fp4_act_quant(src, group)
        assert np.array_equal(got_c.cpu().numpy(), wc)
        assert np.array_equal(got_s.cpu().numpy().view(np.uint32), ws.view(np.uint32))
        stored.append((wc, ws))
    check_close_bf16(bits_of(z), ref.silu_mul_fwd(gb, ub))
    # backward: z recomputed from the stored E2M1 tensors
    gd = ref.fp4_act_dequant(stored[0][0], stored[0][1], n, group)
    ud = ref.fp4_act_dequant(stored[1][0], stored[1][1], n, group)
    z2 = agoq.act_dequant_silu_mul(gc, gs, 4, uc, us, 4, n, group, fp4=True)
    torch.cuda.synchronize()
    got = bits_of(z2)
    assert not np.any((got & 0x7F80) == 0x7F80), "NaN or Inf in the output"
    check_close_bf16(got, ref.silu_mul_fwd(gd, ud))


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("rows,cols", [(3, 128), (64, 4096), (33, 5120), (5, 14336)])
def test_fp4_rmsnorm_forward_with_quantized_input(agoq, ref, rows, cols, group):
    x = wl.act_host(rows, cols, 12000 + rows + cols, "student_t3", max(1, cols // 100), 50.0)
    if rows > 4:
        x[2] = 0
    rng = np.random.default_rng(cols + 5)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x), torch.from_numpy(gamma).cuda(), eps, group, 4, fp4=True)
    torch.cuda.synchronize()
    wc, ws = ref.fp4_act_quant(x, group)
    assert np.array_equal(codes.cpu().numpy(), wc)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    want_y, want_r = ref.rmsnorm_fwd(x, rows, cols, gamma, eps)
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)


# Shapes with enough rows per workgroup for the row kernels' steady loop (refills issued
# without a test) plus a tail of every length: the grid is one or two workgroups per compute
# unit on 14336-wide rows, eight on 4096-wide ones.
MANY_ROWS = [(2048 + 52, 14336, 4), (2048 + 52, 14336, 8), (4096 + 700, 14336, 5), (4096 + 700, 14336, 6),
             (16384 + 1031, 4096, 4), (8192 + 515, 4096, 8), (6 * 768 + 5, 5120, 8),
             # 4096-wide rows take the wavefront-per-row kernels (four rows per workgroup, two
             # workgroups per compute unit): a single row, fewer rows than a workgroup has
             # wavefronts, one row per wavefront with a ragged last workgroup, several rounds
             (1, 4096, 4), (3, 4096, 6), (2048 + 3, 4096, 5), (4096 + 3, 4096, 6), (6144 + 1, 4096, 5),
             (8192 + 7, 4096, 5), (8192 + 2, 4096, 6),
             # 5120-wide rows: ten vectors per lane in the same kernels
             (1024 + 1, 5120, 4), (8192 + 3, 5120, 5), (8192 + 9, 5120, 6), (8192 + 1, 5120, 4),
             # the recompute kernel changes form at 2048 rows (8-bit), 4096 (5/6-bit), 8192 (4-bit)
             (2048 + 5, 4096, 8), (2048 - 1, 4096, 8), (2048 + 1, 5120, 8), (4096 + 1, 5120, 5), (4096 - 1, 4096, 6)]


@pytest.mark.parametrize("rows,cols,bits", MANY_ROWS)
def test_row_kernels_with_many_rows_per_workgroup(agoq, ref, rows, cols, bits):
    group = 128
    x = wl.act_host(rows, cols, 31000 + rows, "normal", max(1, cols // 200), 30.0)
    x[rows // 2] = 0
    rng = np.random.default_rng(rows)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x), torch.from_numpy(gamma).cuda(), eps, group, bits)
    torch.cuda.synchronize()
    wc, ws = ref.act_quant(x, group, bits)
    assert np.array_equal(codes.cpu().numpy(), wc)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    want_y, want_r = ref.rmsnorm_fwd(x, rows, cols, gamma, eps)
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)
    want_y2, want_r2 = ref.act_dequant_rmsnorm(wc, ws, rows, cols, group, bits, gamma, eps)
    y2, r2 = agoq.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, torch.from_numpy(gamma).cuda(), eps)
    torch.cuda.synchronize()
    assert np.allclose(r2.cpu().numpy(), want_r2, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y2), want_y2)


# The wavefront-per-row kernels (4096-wide rows, many rows) at group 64 and on E2M1 codes: the
# forward kernel's stored form bit for bit, both layer outputs to the bar of the fused kernels.
@pytest.mark.parametrize("group,bits,fp4", [(64, 4, False), (64, 6, False), (64, 8, False), (64, 4, True), (128, 4, True)])
def test_wavefront_per_row_kernels_other_groups_and_code_books(agoq, ref, group, bits, fp4):
    rows, cols = 8192 + 5, 4096
    x = wl.act_host(rows, cols, 33000 + group + bits, "student_t3", 40, 50.0)
    x[rows - 2] = 0
    rng = np.random.default_rng(group + bits)
    gamma = (1.0 + 0.2 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    dg = torch.from_numpy(gamma).cuda()
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x), dg, eps, group, bits, fp4=fp4)
    torch.cuda.synchronize()
    wc, ws = ref.fp4_act_quant(x, group) if fp4 else ref.act_quant(x, group, bits)
    assert np.array_equal(codes.cpu().numpy(), wc)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    want_y, want_r = ref.rmsnorm_fwd(x, rows, cols, gamma, eps)
    assert np.allclose(r.cpu().numpy(), want_r, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y), want_y)
    if fp4:
        xd = ref.fp4_act_dequant(wc, ws, rows * cols, group)
        want_y2, want_r2 = ref.rmsnorm_fwd(xd, rows, cols, gamma, eps)
    else:
        want_y2, want_r2 = ref.act_dequant_rmsnorm(wc, ws, rows, cols, group, bits, gamma, eps)
    y2, r2 = agoq.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, dg, eps, fp4=fp4)
    torch.cuda.synchronize()
    assert np.allclose(r2.cpu().numpy(), want_r2, rtol=2e-6, atol=0)
    check_close_bf16(bits_of(y2), want_y2)
