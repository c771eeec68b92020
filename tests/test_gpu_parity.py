"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, bit for bit.

Bar: scales equal as uint32, code bytes equal, dequantized bf16 equal as uint16, reduce
outputs equal in the library's (fixed) summation order.  No tolerance anywhere.
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


def dev_bf16(bits_u16):
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def host_bits(t_bf16):
    return t_bf16.view(torch.int16).cpu().numpy().view(np.uint16)


def same_f32(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


def check_act(agoq, ref, x_bits, group, bits):
    x_bits = np.ascontiguousarray(x_bits).reshape(-1)
    n = x_bits.size
    want_codes, want_scales = ref.act_quant(x_bits, group, bits)
    codes, scales = agoq.act_quant(dev_bf16(x_bits), group, bits)
    torch.cuda.synchronize()
    assert same_f32(scales.cpu().numpy(), want_scales), "scales differ"
    assert np.array_equal(codes.cpu().numpy(), want_codes), "codes differ"
    want_y = ref.act_dequant(want_codes, want_scales, n, group, bits)
    y = agoq.act_dequant(codes, scales, n, group, bits)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(y), want_y), "dequantized values differ"


# ---- config 1 (tiny) ---------------------------------------------------------

def test_tiny_activation_int4_group128(agoq, ref):
    cfg = wl.CONFIGS["tiny"]
    x = wl.act_host(seed=cfg["seed"], **cfg["act"])
    check_act(agoq, ref, x, cfg["group"], cfg["bits"])


def test_tiny_gradient_quant_and_reduce(agoq, ref):
    cfg = wl.CONFIGS["tiny"]
    gc = cfg["grad"]
    group, K, n = cfg["group"], cfg["K"], gc["n"]
    grads = [wl.grad_host(n, seed, gc["sigma"]) for seed in gc["seeds"]]
    pairs = [ref.grad_quant(g, group) for g in grads]
    codes, scales = agoq.grad_quant(torch.from_numpy(grads[0]).cuda(), group)
    torch.cuda.synchronize()
    assert same_f32(scales.cpu().numpy(), pairs[0][1])
    assert np.array_equal(codes.cpu().numpy(), pairs[0][0])
    in_codes = np.stack([p[0] for p in pairs])
    in_scales = np.stack([p[1] for p in pairs])
    want = ref.grad_reduce_requant(in_codes, in_scales, n, group)
    got = agoq.grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(),
                                   n, group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])
    # the fixed-order fp32 sum also sits within 1e-6 (relative to the sum of magnitudes) of binary64
    s64, a64 = ref.grad_reduce_f64(in_codes, in_scales, n, group)
    deq = got[0].cpu().numpy().astype(np.float64) * np.repeat(got[1].cpu().numpy().astype(np.float64), group)
    step = np.repeat(got[1].cpu().numpy().astype(np.float64), group)
    assert np.all(np.abs(deq - s64) <= 0.5 * step * (1 + 2.0 ** -14) + 1e-6 * a64)


# ---- sizes that span several blocks and leave a ragged tail -------------------

@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 3, 64, 65, 8 * 64 + 5, 3 * 8192 // 64 + 7, 40013])
def test_activation_sizes(agoq, ref, bits, group, n_groups):
    rng = np.random.default_rng(1000 + n_groups)
    x = rng.standard_normal(n_groups * group).astype(np.float32)
    x *= (10.0 ** rng.integers(-3, 4, size=x.size)).astype(np.float32)
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    check_act(agoq, ref, xb, group, bits)


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("group", [64, 128])
def test_every_bf16_pattern(agoq, ref, bits, group):
    # all finite bf16 patterns (denormals included), shuffled, plus sorted runs so that
    # some groups are all-tiny (below the 2^-100 rule) and some all-huge
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    pats = pats[((pats >> 7) & 0xFF) != 0xFF]
    rng = np.random.default_rng(7)
    parts = [np.sort(pats), pats[rng.permutation(pats.size)]]
    for scale_exp in (0x0100, 0x0D00, 0x0D80, 0x0E00, 0x3F80, 0x7F00):
        near = (rng.integers(0, 0x200, 4096) + scale_exp - 0x100).astype(np.uint16)
        near = np.where(((near >> 7) & 0xFF) == 0xFF, 0, near)
        parts.append(near | (rng.integers(0, 2, 4096) << 15).astype(np.uint16))
    x = np.concatenate(parts)
    x = x[: x.size // group * group]
    check_act(agoq, ref, x, group, bits)


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_zero_and_tiny_groups(agoq, ref, bits):
    group = 128
    x = np.zeros((6, group), np.uint16)
    x[1] = 0x8000                                   # negative zeros
    x[2, 17] = 0x0D00                               # 2^-101: still stored as zero
    x[3, 17] = 0x0D80                               # 2^-100: quantized
    x[4, :] = 0x0001                                # smallest denormal everywhere
    x[5] = wl.act_host(1, group, 3)[0]
    check_act(agoq, ref, x, group, bits)
    codes, scales = agoq.act_quant(dev_bf16(x.reshape(-1)), group, bits)
    torch.cuda.synchronize()
    s = scales.cpu().numpy()
    assert s[0] == 0 and s[1] == 0 and s[2] == 0 and s[4] == 0 and s[3] > 0 and s[5] > 0
    assert not codes.cpu().numpy()[: 3 * group // 2 if bits != 8 else 3 * group].any()


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("group", [64, 128])
def test_dequant_arbitrary_codes_and_scales(agoq, ref, bits, group):
    # any byte is a legal code (incl. -8 / -128); scales span denormals to large values
    rng = np.random.default_rng(77)
    n_groups = 4099
    n = n_groups * group
    codes = rng.integers(0, 256, size=n * bits // 8).astype(np.uint8)
    scales = (rng.random(n_groups).astype(np.float32) + np.float32(0.5)) * \
        (2.0 ** rng.integers(-140, 100, n_groups)).astype(np.float32)
    scales[::97] = 0.0
    scales[5] = np.float32(1e-45)
    scales = scales.astype(np.float32)
    want = ref.act_dequant(codes, scales, n, group, bits)
    got = agoq.act_dequant(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(), n, group, bits)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(got), want)


# ---- gradients ------------------------------------------------------------------

@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 2, 31, 32, 33, 4 * 32 + 3, 50021])
def test_gradient_quant_sizes(agoq, ref, group, n_groups):
    rng = np.random.default_rng(2000 + n_groups)
    g = (rng.standard_normal(n_groups * group) * 1e-4).astype(np.float32)
    g[rng.random(g.size) < 0.001] *= 100.0
    if n_groups > 8:
        g[group * 2: group * 3] = 0.0                                 # a zero group
        g[group * 3: group * 4] = np.float32(1e-42)                   # denormals only
        g[group * 4: group * 5] *= np.float32(1e-30)                  # tiny but live
        g[group * 5 + 3] = np.float32(3.0e38)                         # near the top of the range
    want = ref.grad_quant(g, group)
    got = agoq.grad_quant(torch.from_numpy(g).cuda(), group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 16, 17, 63, 64])
def test_reduce_requant_chunk_counts(agoq, ref, group, K):
    rng = np.random.default_rng(3000 + K)
    n_groups = 2 * 256 * 16 // group + 3          # two blocks and a ragged tail
    n = n_groups * group
    stride_c = n + 16 * 5
    stride_s = n_groups + 4
    in_codes = rng.integers(-128, 128, size=(K, stride_c)).astype(np.int8)
    in_scales = (rng.random((K, stride_s)) * 1e-5).astype(np.float32)
    in_scales[:, 3] = 0.0                                               # a dead group
    in_scales[0, 4] = np.float32(1e-41)                                 # a denormal scale
    want = ref.grad_reduce_requant(in_codes, in_scales, n, group)
    got = agoq.grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(),
                                   n, group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])


def test_reduce_of_quantized_gradients_with_spikes(agoq, ref):
    group, K, n = 128, 8, 128 * 3001
    grads = [wl.grad_host(n, 500 + k, 1e-4, 0.001, 100.0) for k in range(K)]
    pairs = [ref.grad_quant(g, group) for g in grads]
    in_codes = np.stack([p[0] for p in pairs])
    in_scales = np.stack([p[1] for p in pairs])
    want = ref.grad_reduce_requant(in_codes, in_scales, n, group)
    got = agoq.grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(),
                                   n, group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])
    assert np.all(np.abs(got[0].cpu().numpy().reshape(-1, group).astype(np.int32)).max(axis=1) == 127)


# ---- calling on a side stream, into caller-provided buffers --------------------

def test_side_stream_and_preallocated_outputs(agoq, ref):
    group, bits = 128, 4
    x = wl.act_host(64, 1024, 9, outlier_channels=5, outlier_scale=30.0)
    xd = dev_bf16(x.reshape(-1))
    codes = torch.zeros(x.size // 2, dtype=torch.uint8, device="cuda")
    scales = torch.zeros(x.size // group, dtype=torch.float32, device="cuda")
    y = torch.zeros(x.size, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        agoq.act_quant(xd, group, bits, codes=codes, scales=scales)
        agoq.act_dequant(codes, scales, x.size, group, bits, out=y)
    st.synchronize()
    wc, ws = ref.act_quant(x, group, bits)
    assert np.array_equal(codes.cpu().numpy(), wc) and same_f32(scales.cpu().numpy(), ws)
    assert np.array_equal(host_bits(y), ref.act_dequant(wc, ws, x.size, group, bits))


# ---- error codes: nothing is launched, outputs stay untouched -------------------

def test_error_codes(agoq):
    import ctypes
    L = agoq.load_library()
    x = torch.zeros(1024, dtype=torch.bfloat16, device="cuda")
    codes = torch.full((1024,), 7, dtype=torch.uint8, device="cuda")
    scales = torch.full((16,), 3.0, dtype=torch.float32, device="cuda")
    P = ctypes.c_void_p
    px, pc, ps = P(x.data_ptr()), P(codes.data_ptr()), P(scales.data_ptr())
    assert L.agoq_act_quant(None, 1024, 128, 4, pc, ps, None) == 1
    assert L.agoq_act_quant(px, 1024, 128, 7, pc, ps, None) == 2
    assert L.agoq_act_quant(px, 1024, 32, 4, pc, ps, None) == 3
    assert L.agoq_act_quant(px, 1000, 128, 4, pc, ps, None) == 4
    assert L.agoq_act_quant(px, 0, 128, 4, pc, ps, None) == 4
    assert L.agoq_act_quant(P(x.data_ptr() + 2), 512, 128, 4, pc, ps, None) == 5
    assert L.agoq_act_dequant(pc, ps, 1024, 128, 3, px, None) == 2
    assert L.agoq_act_dequant(pc, None, 1024, 128, 4, px, None) == 1
    g = torch.zeros(1024, dtype=torch.float32, device="cuda")
    pg = P(g.data_ptr())
    assert L.agoq_grad_quant(pg, 1024, 100, pc, ps, None) == 3
    assert L.agoq_grad_quant(pg, 1024 + 64, 128, pc, ps, None) == 4
    assert L.agoq_grad_reduce_requant(pc, 1024, ps, 8, 0, 1024, 128, pc, ps, None) == 6
    assert L.agoq_grad_reduce_requant(pc, 1024, ps, 8, 65, 1024, 128, pc, ps, None) == 6
    assert L.agoq_grad_reduce_requant(pc, 512, ps, 8, 2, 1024, 128, pc, ps, None) == 4
    assert L.agoq_grad_reduce_requant(pc, 1024, ps, 4, 2, 1024, 128, pc, ps, None) == 4
    assert L.agoq_grad_reduce_requant(pc, 1032, ps, 8, 2, 1024, 128, pc, ps, None) == 5
    assert L.agoq_grad_reduce_requant(pc, 1024, P(scales.data_ptr() + 4), 8, 2, 1024, 128, pc, ps, None) == 5
    torch.cuda.synchronize()
    assert bool((codes == 7).all()) and bool((scales == 3.0).all())
    with pytest.raises(agoq.AgoqError):
        agoq.act_quant(x, 128, 7)
    with pytest.raises(TypeError):
        agoq.act_quant(x.float(), 128, 4)
    with pytest.raises(TypeError):
        agoq.act_quant(x.cpu(), 128, 4)


# ---- local accumulation into the stored 8-bit gradient, and int8 -> fp32 dequantize ----

@pytest.mark.parametrize("as_bf16", [False, True])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 17, 4 * 32 + 3, 30011])
def test_gradient_accumulate(agoq, ref, group, n_groups, as_bf16):
    rng = np.random.default_rng(4000 + n_groups)
    n = n_groups * group
    base = wl.grad_host(n, 4100 + n_groups, 1e-4, 0.001, 100.0)
    main_c, main_s = ref.grad_quant(base, group)
    g32 = wl.grad_host(n, 4200 + n_groups, 1e-4, 0.001, 100.0)
    if n_groups > 8:
        g32[group * 2: group * 3] = 0.0
        main_c[group * 2: group * 3] = 0                      # 0 + 0: a dead group
        g32[group * 5: group * 6] = -ref.grad_dequant(main_c, main_s, group)[group * 5: group * 6]
    if as_bf16:
        t = torch.from_numpy(g32).to(torch.bfloat16)
        g_host = t.view(torch.int16).numpy().view(np.uint16)
        g_dev = t.cuda()
    else:
        g_host = g32
        g_dev = torch.from_numpy(g32).cuda()
    want = ref.grad_accumulate(main_c, main_s, g_host, group)
    d_c, d_s = torch.from_numpy(main_c).cuda(), torch.from_numpy(main_s).cuda()
    out_c = torch.empty_like(d_c)
    out_s = torch.empty_like(d_s)
    agoq.grad_accumulate(d_c, d_s, g_dev, group, out_codes=out_c, out_scales=out_s)
    torch.cuda.synchronize()
    assert same_f32(out_s.cpu().numpy(), want[1])
    assert np.array_equal(out_c.cpu().numpy(), want[0])
    assert np.array_equal(d_c.cpu().numpy(), main_c)          # inputs untouched
    # in place: the stored gradient is overwritten with the same result
    agoq.grad_accumulate(d_c, d_s, g_dev, group)
    torch.cuda.synchronize()
    assert same_f32(d_s.cpu().numpy(), want[1])
    assert np.array_equal(d_c.cpu().numpy(), want[0])


def test_gradient_accumulate_over_micro_batches_tracks_the_sum(agoq, ref):
    # eight micro-batches accumulated in place; oracle and GPU stay bit-identical, and the
    # stored gradient stays within the quantization steps of the true fp32 sum
    group, n = 128, 128 * 2048
    d_c = torch.zeros(n, dtype=torch.int8, device="cuda")
    d_s = torch.zeros(n // group, dtype=torch.float32, device="cuda")
    h_c, h_s = np.zeros(n, np.int8), np.zeros(n // group, np.float32)
    total = np.zeros(n, np.float64)
    slack = np.zeros(n // group, np.float64)
    for mb in range(8):
        g = wl.grad_host(n, 4300 + mb, 1e-4, 0.001, 100.0)
        total += g
        agoq.grad_accumulate(d_c, d_s, torch.from_numpy(g).cuda(), group)
        h_c, h_s = ref.grad_accumulate(h_c, h_s, g, group)
        slack += 0.5 * h_s.astype(np.float64) * 1.001
    torch.cuda.synchronize()
    assert np.array_equal(d_c.cpu().numpy(), h_c) and same_f32(d_s.cpu().numpy(), h_s)
    deq = agoq.grad_dequant(d_c, d_s, group)
    torch.cuda.synchronize()
    assert np.array_equal(deq.cpu().numpy(), ref.grad_dequant(h_c, h_s, group))
    assert np.all(np.abs(deq.cpu().numpy().astype(np.float64) - total) <= np.repeat(slack, group) + 1e-12)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 5, 8 * 512 * 4 // 32 + 3, 70001])
def test_gradient_dequant(agoq, ref, group, n_groups):
    rng = np.random.default_rng(4400 + n_groups)
    n = n_groups * group
    codes = rng.integers(-128, 128, size=n).astype(np.int8)
    scales = (rng.random(n_groups).astype(np.float32) + np.float32(0.5)) * \
        (2.0 ** rng.integers(-140, 100, n_groups)).astype(np.float32)
    scales[::53] = 0.0
    want = ref.grad_dequant(codes, scales.astype(np.float32), group)
    got = agoq.grad_dequant(torch.from_numpy(codes).cuda(), torch.from_numpy(scales.astype(np.float32)).cuda(), group)
    torch.cuda.synchronize()
    assert same_f32(got.cpu().numpy(), want)


def test_accumulate_and_dequant_error_codes(agoq):
    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    c = torch.zeros(1024, dtype=torch.int8, device="cuda")
    s = torch.zeros(8, dtype=torch.float32, device="cuda")
    g = torch.zeros(1024, dtype=torch.float32, device="cuda")
    pc, ps, pg = P(c.data_ptr()), P(s.data_ptr()), P(g.data_ptr())
    assert L.agoq_grad_accumulate(pc, ps, None, 0, 1024, 128, pc, ps, None) == 1
    assert L.agoq_grad_accumulate(pc, ps, pg, 0, 1024, 96, pc, ps, None) == 3
    assert L.agoq_grad_accumulate(pc, ps, pg, 0, 1000, 128, pc, ps, None) == 4
    assert L.agoq_grad_accumulate(pc, ps, P(g.data_ptr() + 4), 0, 512, 128, pc, ps, None) == 5
    assert L.agoq_grad_dequant(pc, None, 1024, 128, pg, None) == 1
    assert L.agoq_grad_dequant(pc, ps, 1024, 32, pg, None) == 3
    assert L.agoq_grad_dequant(pc, ps, -128, 128, pg, None) == 4


def test_gradient_codes_dequantize_to_bf16_through_the_activation_call(agoq, ref):
    """int8 gradient codes and 8-bit activation codes share a layout: the activation
    dequantize gives bf16(code * scale) of a stored gradient."""
    group, n = 128, 128 * 7001
    g = wl.grad_host(n, 77, 1e-4, 0.001, 100.0)
    codes, scales = agoq.grad_quant(torch.from_numpy(g).cuda(), group)
    y = agoq.act_dequant(codes.view(torch.uint8), scales, n, group, 8)
    torch.cuda.synchronize()
    wc, ws = ref.grad_quant(g, group)
    f32 = ref.grad_dequant(wc, ws, group)
    want = torch.from_numpy(f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(host_bits(y), want)
    assert np.array_equal(host_bits(y), ref.act_dequant(wc.view(np.uint8), ws, n, group, 8))
