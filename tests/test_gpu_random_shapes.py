"""GPU parity on seeded random shapes: sizes, widths, group sizes, chunk counts and strides
drawn at random (a fixed seed per case), every call compared bit for bit with the oracle.
Sizes are drawn around the tile sizes of the kernels (a workgroup handles 256 to 4096
16-byte vectors) as well as uniformly, so whole tiles, ragged tails and tensors smaller than
one tile all occur."""
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


def dev_bf16(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def same(a, b):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def draw_groups(rng, group, per_lane):
    """A number of groups: small, or near a multiple of a tile of 128..1024 lanes."""
    kind = rng.integers(0, 3)
    if kind == 0:
        return int(rng.integers(1, 40))
    if kind == 1:
        return int(rng.integers(40, 6000))
    lanes = int(rng.choice([128, 256, 512, 1024])) * int(rng.choice([1, 2, 4]))
    tile_groups = max(lanes * per_lane // group, 1)
    return max(1, tile_groups * int(rng.integers(1, 9)) + int(rng.integers(-2, 3)))


def random_bf16(rng, n):
    """Values over many magnitudes, exact zeros, and a few dead groups' worth of tiny numbers."""
    x = rng.standard_normal(n).astype(np.float32) * np.exp2(rng.integers(-20, 20, n)).astype(np.float32)
    x[rng.random(n) < 0.05] = 0.0
    bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    return bits


@pytest.mark.parametrize("case", range(40))
def test_activation_calls(agoq, ref, case):
    rng = np.random.default_rng(20000 + case)
    group = int(rng.choice([64, 128]))
    bits = int(rng.choice([4, 5, 6, 8]))
    n = group * draw_groups(rng, group, 8)
    x = random_bf16(rng, n)
    if rng.random() < 0.3:
        g = int(rng.integers(0, n // group))
        x[g * group:(g + 1) * group] = 0                          # a dead group
    wc, ws = ref.act_quant(x, group, bits)
    c, s = agoq.act_quant(dev_bf16(x), group, bits)
    torch.cuda.synchronize()
    assert same(s.cpu().numpy(), ws) and same(c.cpu().numpy(), wc), (group, bits, n)
    y = agoq.act_dequant(c, s, n, group, bits)
    torch.cuda.synchronize()
    assert same(host_bits(y), ref.act_dequant(wc, ws, n, group, bits)), (group, bits, n)
    if bits == 4:
        fc, fs = ref.fp4_act_quant(x, group)
        c, s = agoq.fp4_act_quant(dev_bf16(x), group)
        y = agoq.fp4_act_dequant(c, s, n, group)
        torch.cuda.synchronize()
        assert same(s.cpu().numpy(), fs) and same(c.cpu().numpy(), fc), (group, n)
        assert same(host_bits(y), ref.fp4_act_dequant(fc, fs, n, group)), (group, n)


@pytest.mark.parametrize("case", range(12))
def test_layer_calls(agoq, ref, case):
    rng = np.random.default_rng(21000 + case)
    group = int(rng.choice([64, 128]))
    count = int(rng.integers(1, 9))
    widths = [int(b) for b in rng.choice([4, 5, 6, 8], count)]
    xs = [random_bf16(rng, group * draw_groups(rng, group, 8)) for _ in range(count)]
    wants = [ref.act_quant(x, group, b) for x, b in zip(xs, widths)]
    codes, scales = agoq.act_quant_layer([dev_bf16(x) for x in xs], group, widths)
    torch.cuda.synchronize()
    for c, s, (wc, ws) in zip(codes, scales, wants):
        assert same(c.cpu().numpy(), wc) and same(s.cpu().numpy(), ws)
    ys = agoq.act_dequant_layer(codes, scales, [x.size for x in xs], group, widths)
    torch.cuda.synchronize()
    for y, x, b, (wc, ws) in zip(ys, xs, widths, wants):
        assert same(host_bits(y), ref.act_dequant(wc, ws, x.size, group, b))


@pytest.mark.parametrize("case", range(30))
def test_gradient_calls(agoq, ref, case):
    rng = np.random.default_rng(22000 + case)
    group = int(rng.choice([64, 128]))
    fp8 = bool(rng.integers(0, 2))
    n = group * draw_groups(rng, group, 16)
    K = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 33, 64]))
    sigma = float(np.exp2(rng.integers(-30, 10)))
    quant = ref.fp8_grad_quant if fp8 else ref.grad_quant
    gq = agoq.fp8_grad_quant if fp8 else agoq.grad_quant
    g0 = wl.grad_host(n, 3000 + case, sigma, 0.01, 50.0)
    wc, ws = quant(g0, group)
    c, s = gq(torch.from_numpy(g0).cuda(), group)
    torch.cuda.synchronize()
    assert same(c.cpu().numpy(), wc) and same(s.cpu().numpy(), ws), (group, fp8, n)
    dq = agoq.fp8_grad_dequant if fp8 else agoq.grad_dequant
    rdq = ref.fp8_grad_dequant if fp8 else ref.grad_dequant
    out = dq(c, s, group)
    torch.cuda.synchronize()
    assert same(out.cpu().numpy(), rdq(wc, ws, group))
    # K chunks in one buffer with padded strides; chunk magnitudes differ by powers of two
    stride_c = n + 16 * int(rng.integers(0, 9))
    stride_s = n // group + 4 * int(rng.integers(0, 5))
    in_codes = np.zeros((K, stride_c), wc.dtype)
    in_scales = np.zeros((K, stride_s), np.float32)
    for k in range(K):
        ck, sk = quant(wl.grad_host(n, 4000 + 70 * case + k, sigma * float(np.exp2(rng.integers(-3, 4))), 0.01, 50.0), group)
        in_codes[k, :n] = ck
        in_scales[k, :n // group] = sk
    in_codes[:, n:] = 77                                       # padding must never be read as data
    in_scales[:, n // group:] = 1e30
    red = agoq.fp8_grad_reduce_requant if fp8 else agoq.grad_reduce_requant
    rred = ref.fp8_grad_reduce_requant if fp8 else ref.grad_reduce_requant
    want_c, want_s = rred(in_codes, in_scales, n, group)
    got_c, got_s = red(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(), n, group)
    torch.cuda.synchronize()
    assert same(got_s.cpu().numpy(), want_s) and same(got_c.cpu().numpy(), want_c), (group, fp8, n, K)
    # accumulate a new micro-batch gradient onto the reduced one, in place
    as_bf16 = bool(rng.integers(0, 2))
    g_new = wl.grad_host(n, 5000 + case, sigma, 0.01, 50.0)
    g_dev = torch.from_numpy(g_new)
    g_host = g_new
    if as_bf16:
        g_dev = g_dev.to(torch.bfloat16)
        g_host = g_dev.view(torch.int16).numpy().view(np.uint16)
    racc = ref.fp8_grad_accumulate if fp8 else ref.grad_accumulate
    acc = agoq.fp8_grad_accumulate if fp8 else agoq.grad_accumulate
    a_c, a_s = racc(want_c, want_s, g_host, group)
    acc(got_c, got_s, g_dev.cuda(), group)
    torch.cuda.synchronize()
    assert same(got_s.cpu().numpy(), a_s) and same(got_c.cpu().numpy(), a_c), (group, fp8, n, as_bf16)
