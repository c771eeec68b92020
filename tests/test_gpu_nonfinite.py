"""GPU parity on tensors that hold Inf and NaN values.

Rule (a reading; the paper is silent): a group that holds a non-finite value -- in the tensor
being quantized or in the fp32 sums of the reduce / accumulation -- stores scale = quiet NaN
(bits 0x7FC00000) and all-zero codes, so the whole group reads back as NaN.  Codes and scales
are compared bit for bit with the oracle's.  Dequantized values are compared bit for bit
where the oracle's value is not a NaN and must be NaNs where it is one: which NaN comes out
of a conversion is not part of the contract.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from test_gpu_recompute import check_close_bf16

pytestmark = pytest.mark.gpu

QNAN = 0x7FC00000
BF16_POISONS = (0x7F80, 0xFF80, 0x7FC0, 0x7FFF, 0xFFC1, 0x7F81)
F32_POISONS = (0x7F800000, 0xFF800000, 0x7FC00000, 0x7FC000FF, 0xFFFFFFFF, 0x7F800001, 0x7FBFFFFF)


@pytest.fixture(scope="module")
def agoq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_00539_amd as lib
    lib.load_library()
    return lib


def dev_bf16(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t_bf16):
    return t_bf16.view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_is_nan(bits):
    bits = np.asarray(bits, np.uint16)
    return ((bits & 0x7F80) == 0x7F80) & ((bits & 0x007F) != 0)


def same_bits(a, b):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def same_bf16_up_to_nan(got, want):
    nan = bf16_is_nan(want)
    return bool(bf16_is_nan(got[nan]).all()) and np.array_equal(got[~nan], want[~nan])


def same_f32_up_to_nan(got, want):
    nan = np.isnan(want)
    return bool(np.isnan(got[nan]).all()) and np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def poisoned_act(rows, cols, seed, group, rng, n_poison):
    x = wl.act_host(rows, cols, seed, outlier_channels=3, outlier_scale=20.0).reshape(-1).copy()
    pos = rng.choice(x.size, n_poison, replace=False)
    pos[0], pos[1], pos[2] = 0, x.size - 1, group * 5 + group - 1     # first, last, end of a group
    x[pos] = np.array(BF16_POISONS, np.uint16)[rng.integers(0, len(BF16_POISONS), n_poison)]
    return x, np.unique(pos // group)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_activation_quantize_and_dequantize(agoq, ref, bits, group):
    rng = np.random.default_rng(bits * 1000 + group)
    rows, cols = 203, 1408                                # several tiles and a ragged last one
    x, bad = poisoned_act(rows, cols, 500 + bits, group, rng, 40)
    want_c, want_s = ref.act_quant(x, group, bits)
    assert np.all(want_s.view(np.uint32)[bad] == QNAN) and np.isfinite(np.delete(want_s, bad)).all()
    codes, scales = agoq.act_quant(dev_bf16(x), group, bits)
    torch.cuda.synchronize()
    assert same_bits(scales.cpu().numpy(), want_s)
    assert same_bits(codes.cpu().numpy(), want_c)
    want_y = ref.act_dequant(want_c, want_s, x.size, group, bits)
    y = agoq.act_dequant(codes, scales, x.size, group, bits)
    torch.cuda.synchronize()
    got_y = host_bits(y)
    assert same_bf16_up_to_nan(got_y, want_y)
    assert bf16_is_nan(got_y.reshape(-1, group)[bad]).all()
    assert not bf16_is_nan(np.delete(got_y.reshape(-1, group), bad, axis=0)).any()


@pytest.mark.parametrize("group", [64, 128])
def test_e2m1_activation(agoq, ref, group):
    rng = np.random.default_rng(group)
    x, bad = poisoned_act(120, 1152, 77, group, rng, 25)
    want_c, want_s = ref.fp4_act_quant(x, group)
    codes, scales = agoq.fp4_act_quant(dev_bf16(x), group)
    torch.cuda.synchronize()
    assert same_bits(scales.cpu().numpy(), want_s)
    assert same_bits(codes.cpu().numpy(), want_c)
    y = agoq.fp4_act_dequant(codes, scales, x.size, group)
    torch.cuda.synchronize()
    assert same_bf16_up_to_nan(host_bits(y), ref.fp4_act_dequant(want_c, want_s, x.size, group))


def test_layer_launches(agoq, ref):
    group = 128
    rng = np.random.default_rng(3)
    shapes = [(64, 1024), (33, 1152), (64, 1024), (40, 3584), (40, 3584)]
    widths = [8, 4, 6, 5, 4]
    xs, wants = [], []
    for i, (r, c) in enumerate(shapes):
        x, _ = poisoned_act(r, c, 900 + i, group, rng, 12)
        xs.append(x)
        wants.append(ref.act_quant(x, group, widths[i]))
    codes, scales = agoq.act_quant_layer([dev_bf16(x) for x in xs], group, widths)
    torch.cuda.synchronize()
    for c, s, (wc, ws) in zip(codes, scales, wants):
        assert same_bits(c.cpu().numpy(), wc) and same_bits(s.cpu().numpy(), ws)
    ys = agoq.act_dequant_layer(codes, scales, [x.size for x in xs], group, widths)
    torch.cuda.synchronize()
    for y, x, b, (wc, ws) in zip(ys, xs, widths, wants):
        assert same_bf16_up_to_nan(host_bits(y), ref.act_dequant(wc, ws, x.size, group, b))


def poisoned_grad(n, seed, group, rng, n_poison):
    g = wl.grad_host(n, seed, 1e-3, 0.001, 100.0).copy()
    pos = rng.choice(n, n_poison, replace=False)
    pos[0], pos[1] = 0, n - 1
    g.view(np.uint32)[pos] = np.array(F32_POISONS, np.uint32)[rng.integers(0, len(F32_POISONS), n_poison)]
    return g, np.unique(pos // group)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("fp8", [False, True])
def test_gradient_store_and_dequantize(agoq, ref, fp8, group):
    rng = np.random.default_rng(11 + group)
    n = group * 4099
    g, bad = poisoned_grad(n, 31, group, rng, 30)
    quant, dequant = (agoq.fp8_grad_quant, agoq.fp8_grad_dequant) if fp8 else (agoq.grad_quant, agoq.grad_dequant)
    rquant, rdequant = (ref.fp8_grad_quant, ref.fp8_grad_dequant) if fp8 else (ref.grad_quant, ref.grad_dequant)
    want_c, want_s = rquant(g, group)
    assert np.all(want_s.view(np.uint32)[bad] == QNAN)
    codes, scales = quant(torch.from_numpy(g).cuda(), group)
    torch.cuda.synchronize()
    assert same_bits(scales.cpu().numpy(), want_s)
    assert same_bits(codes.cpu().numpy(), want_c)
    out = dequant(codes, scales, group)
    torch.cuda.synchronize()
    assert same_f32_up_to_nan(out.cpu().numpy(), rdequant(want_c, want_s, group))


@pytest.mark.parametrize("K", [1, 2, 3, 4, 8, 16])
@pytest.mark.parametrize("fp8", [False, True])
def test_reduce(agoq, ref, fp8, K):
    """Chunks whose senders saw non-finite gradients (NaN scales), and full-scale terms that
    are finite one by one but overflow binary32 when summed."""
    group = 128
    n = group * 3001
    rng = np.random.default_rng(100 + K)
    rquant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    pairs = []
    for k in range(K):
        g, _ = poisoned_grad(n, 40 + k, group, rng, 6)
        pairs.append(rquant(g, group))
    codes = np.stack([p[0] for p in pairs])
    scales = np.stack([p[1] for p in pairs])
    big = np.float32(2.0 ** 127) / np.float32(448.0 if fp8 else 127.0) * np.float32(1.5)
    full = 0x7E if fp8 else 127
    for grp in (7, 1500, 3000):                             # overflow: K >= 2 only
        for k in range(min(K, 2)):
            scales[k, grp] = big
            codes[k, grp * group + 5] = full
    reduce_ = ref.fp8_grad_reduce_requant if fp8 else ref.grad_reduce_requant
    want_c, want_s = reduce_(codes, scales, n, group)
    assert np.isnan(want_s).sum() >= 4 and np.isfinite(want_s).sum() > 2900
    if K >= 2:
        assert np.all(want_s.view(np.uint32)[[7, 1500, 3000]] == QNAN)
    call = agoq.fp8_grad_reduce_requant if fp8 else agoq.grad_reduce_requant
    got_c, got_s = call(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(), n, group)
    torch.cuda.synchronize()
    assert same_bits(got_s.cpu().numpy(), want_s)
    assert same_bits(got_c.cpu().numpy(), want_c)


@pytest.mark.parametrize("addend", ["f32", "bf16"])
@pytest.mark.parametrize("fp8", [False, True])
def test_accumulate(agoq, ref, fp8, addend):
    group = 64
    n = group * 5003
    rng = np.random.default_rng(17)
    g_main, _ = poisoned_grad(n, 61, group, rng, 9)         # stored gradient with NaN groups
    rquant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    main_c, main_s = rquant(g_main, group)
    g_new, _ = poisoned_grad(n, 62, group, rng, 9)
    if addend == "bf16":
        g_in = torch.from_numpy(g_new).to(torch.bfloat16)   # Inf stays Inf, NaN stays NaN
        g_host = g_in.view(torch.int16).numpy().view(np.uint16)
    else:
        g_in = torch.from_numpy(g_new)
        g_host = g_new
    racc = ref.fp8_grad_accumulate if fp8 else ref.grad_accumulate
    want_c, want_s = racc(main_c, main_s, g_host, group)
    assert 9 <= np.isnan(want_s).sum() <= 18
    d_c, d_s = torch.from_numpy(main_c).cuda(), torch.from_numpy(main_s).cuda()
    call = agoq.fp8_grad_accumulate if fp8 else agoq.grad_accumulate
    call(d_c, d_s, g_in.cuda(), group)                      # in place
    torch.cuda.synchronize()
    assert same_bits(d_s.cpu().numpy(), want_s)
    assert same_bits(d_c.cpu().numpy(), want_c)


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_fused_calls_store_the_same_codes_and_propagate(agoq, ref, bits):
    """Forward side: the stored codes and scales follow the rule.  Backward side: a row of
    RMSNorm that holds a NaN group is NaN all over (its mean square is), SiLU & Multiply is
    NaN exactly in the poisoned groups; everything else stays within the usual tolerance."""
    group, rows, cols = 128, 96, 1024
    rng = np.random.default_rng(bits)
    x, bad = poisoned_act(rows, cols, 70 + bits, group, rng, 5)
    gamma = (1.0 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    want_c, want_s = ref.act_quant(x, group, bits)
    y, r, codes, scales = agoq.rmsnorm_fwd_quant(dev_bf16(x).view(rows, cols), torch.from_numpy(gamma).cuda(),
                                                 1e-5, group, bits)
    torch.cuda.synchronize()
    assert same_bits(codes.cpu().numpy(), want_c) and same_bits(scales.cpu().numpy(), want_s)
    bad_rows = np.unique(bad // (cols // group))
    good_rows = np.setdiff1d(np.arange(rows), bad_rows)
    want_y, want_r = ref.act_dequant_rmsnorm(want_c, want_s, rows, cols, group, bits, gamma, 1e-5)
    y2, r2 = agoq.act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, torch.from_numpy(gamma).cuda(), 1e-5)
    torch.cuda.synchronize()
    got = host_bits(y2).reshape(rows, cols)
    assert bf16_is_nan(got[bad_rows]).all() and np.isnan(r2.cpu().numpy()[bad_rows]).all()
    assert bf16_is_nan(want_y.reshape(rows, cols)[bad_rows]).all()
    assert not bf16_is_nan(got[good_rows]).any()
    check_close_bf16(got[good_rows].reshape(-1), want_y.reshape(rows, cols)[good_rows].reshape(-1))
    # SiLU & Multiply on (x as gate, a clean up tensor)
    up = wl.act_host(rows, cols, 99).reshape(-1)
    uc, us = ref.act_quant(up, group, 4)
    want_z = ref.act_dequant_silu_mul(want_c, want_s, bits, uc, us, 4, rows * cols, group)
    z = agoq.act_dequant_silu_mul(codes, scales, bits, torch.from_numpy(uc).cuda(), torch.from_numpy(us).cuda(), 4,
                                  rows * cols, group)
    torch.cuda.synchronize()
    gz = host_bits(z).reshape(-1, group)
    wz = want_z.reshape(-1, group)
    assert bf16_is_nan(gz[bad]).all() and bf16_is_nan(wz[bad]).all()
    keep = np.setdiff1d(np.arange(gz.shape[0]), bad)
    assert not bf16_is_nan(gz[keep]).any()
    check_close_bf16(gz[keep].reshape(-1), wz[keep].reshape(-1))
