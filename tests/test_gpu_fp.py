"""GPU parity for the floating-point code books (E2M1 activations, E4M3 gradients), bit for bit."""
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


def same_f32(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


def check_fp4(agoq, ref, x_bits, group):
    x_bits = np.ascontiguousarray(x_bits).reshape(-1)
    n = x_bits.size
    wc, ws = ref.fp4_act_quant(x_bits, group)
    codes, scales = agoq.fp4_act_quant(dev_bf16(x_bits), group)
    torch.cuda.synchronize()
    assert same_f32(scales.cpu().numpy(), ws), "scales differ"
    assert np.array_equal(codes.cpu().numpy(), wc), "codes differ"
    y = agoq.fp4_act_dequant(codes, scales, n, group)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(y), ref.fp4_act_dequant(wc, ws, n, group)), "dequantized values differ"


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 3, 65, 8 * 64 + 5, 40013])
def test_fp4_activation_sizes(agoq, ref, group, n_groups):
    rng = np.random.default_rng(5000 + n_groups)
    x = rng.standard_normal(n_groups * group).astype(np.float32)
    x *= (10.0 ** rng.integers(-3, 4, size=x.size)).astype(np.float32)
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    check_fp4(agoq, ref, xb, group)


@pytest.mark.parametrize("group", [64, 128])
def test_fp4_every_bf16_pattern_and_dead_groups(agoq, ref, group):
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    pats = pats[((pats >> 7) & 0xFF) != 0xFF]
    rng = np.random.default_rng(8)
    dead = np.zeros(4 * group, np.uint16)
    dead[::2] = 0x8000                                   # negative zeros
    dead[group + 3] = 0x0D00                             # 2^-101
    dead[2 * group: 3 * group] = 0x8001                  # negative denormals
    x = np.concatenate([np.sort(pats), pats[rng.permutation(pats.size)], dead])
    x = x[: x.size // group * group]
    check_fp4(agoq, ref, x, group)


@pytest.mark.parametrize("group", [64, 128])
def test_fp4_dequant_any_codes(agoq, ref, group):
    rng = np.random.default_rng(9)
    n_groups = 4099
    n = n_groups * group
    codes = rng.integers(0, 256, size=n // 2).astype(np.uint8)          # every nibble incl. -0
    scales = ((rng.random(n_groups).astype(np.float32) + np.float32(0.5)) *
              (2.0 ** rng.integers(-140, 100, n_groups)).astype(np.float32)).astype(np.float32)
    scales[::97] = 0.0
    want = ref.fp4_act_dequant(codes, scales, n, group)
    got = agoq.fp4_act_dequant(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(), n, group)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(got), want)


@pytest.mark.parametrize("name", ["A", "F"])
def test_fp4_llama8b_activations_full_size(agoq, ref, name):
    cfg = wl.CONFIGS["llama8b_act"]
    shape = cfg["acts"][name]
    x = wl.act_device(shape["rows"], shape["cols"], cfg["seed"] + 7, cfg["dist"],
                      wl.n_outlier_channels(shape["cols"], cfg["outlier_frac"]), cfg["outlier_scale"])
    check_fp4(agoq, ref, host_bits(x.reshape(-1)), cfg["group"])


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 2, 33, 4 * 32 + 3, 50021])
def test_fp8_gradient_store_and_dequant(agoq, ref, group, n_groups):
    rng = np.random.default_rng(6000 + n_groups)
    g = (rng.standard_normal(n_groups * group) * 1e-4).astype(np.float32)
    g[rng.random(g.size) < 0.001] *= 100.0
    if n_groups > 8:
        g[group * 2: group * 3] = 0.0
        g[group * 2: group * 3: 2] = -0.0                                # a dead group with signed zeros
        g[group * 3: group * 4] = np.float32(-1e-42)                     # negative denormals only
        g[group * 4: group * 5] *= np.float32(1e-30)
        g[group * 5 + 3] = np.float32(3.0e38)
    wc, ws = ref.fp8_grad_quant(g, group)
    codes, scales = agoq.fp8_grad_quant(torch.from_numpy(g).cuda(), group)
    torch.cuda.synchronize()
    assert same_f32(scales.cpu().numpy(), ws)
    assert np.array_equal(codes.cpu().numpy(), wc)
    out = agoq.fp8_grad_dequant(codes, scales, group)
    torch.cuda.synchronize()
    assert same_f32(out.cpu().numpy(), ref.fp8_grad_dequant(wc, ws, group))


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 16, 17, 64])
def test_fp8_reduce_requant_chunk_counts(agoq, ref, group, K):
    rng = np.random.default_rng(7000 + K)
    n_groups = 2 * 512 * 16 // group + 3
    n = n_groups * group
    stride_c, stride_s = n + 16 * 5, n_groups + 3
    in_codes = rng.integers(0, 256, size=(K, stride_c)).astype(np.uint8)
    in_codes[(in_codes & 0x7F) == 0x7F] = 0x35                            # no NaN codes
    in_scales = (rng.random((K, stride_s)) * 1e-5).astype(np.float32)
    in_scales[:, 3] = 0.0                                                 # a dead group (signed zeros inside)
    want = ref.fp8_grad_reduce_requant(in_codes, in_scales, n, group)
    got = agoq.fp8_grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(),
                                       n, group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])


def test_fp8_llama8b_gradient_shard_store_and_reduce(agoq, ref):
    cfg = wl.CONFIGS["llama8b_grad"]
    group, K = cfg["group"], cfg["K"]
    n = cfg["n"] // K                                                     # one GPU's shard of the layer
    pairs = []
    for k in range(K):
        g = wl.grad_device(n, cfg["seed"] + 50 + k, cfg["sigma"], cfg["spike_frac"], cfg["spike_scale"])
        gh = g.cpu().numpy()
        pairs.append(ref.fp8_grad_quant(gh, group))
        if k == 0:
            codes, scales = agoq.fp8_grad_quant(g, group)
            torch.cuda.synchronize()
            assert same_f32(scales.cpu().numpy(), pairs[0][1]) and np.array_equal(codes.cpu().numpy(), pairs[0][0])
    in_codes = np.stack([p[0] for p in pairs])
    in_scales = np.stack([p[1] for p in pairs])
    want = ref.fp8_grad_reduce_requant(in_codes, in_scales, n, group)
    got = agoq.fp8_grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(),
                                       n, group)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1]) and np.array_equal(got[0].cpu().numpy(), want[0])
    assert np.all((want[0].reshape(-1, group) & 0x7F).max(axis=1)[want[1] > 0] == 126)   # full scale, never beyond


def test_fp_error_codes(agoq):
    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    x = torch.zeros(1024, dtype=torch.bfloat16, device="cuda")
    c = torch.full((1024,), 7, dtype=torch.uint8, device="cuda")
    s = torch.full((16,), 3.0, dtype=torch.float32, device="cuda")
    g = torch.zeros(1024, dtype=torch.float32, device="cuda")
    px, pc, ps, pg = (P(t.data_ptr()) for t in (x, c, s, g))
    assert L.agoq_fp4_act_quant(None, 1024, 128, pc, ps, None) == 1
    assert L.agoq_fp4_act_quant(px, 1024, 32, pc, ps, None) == 3
    assert L.agoq_fp4_act_quant(px, 1000, 128, pc, ps, None) == 4
    assert L.agoq_fp4_act_dequant(pc, ps, 1024, 128, P(x.data_ptr() + 2), None) == 5
    assert L.agoq_fp8_grad_quant(pg, 1024, 100, pc, ps, None) == 3
    assert L.agoq_fp8_grad_dequant(pc, None, 1024, 128, pg, None) == 1
    assert L.agoq_fp8_grad_reduce_requant(pc, 1024, ps, 8, 0, 1024, 128, pc, ps, None) == 6
    assert L.agoq_fp8_grad_reduce_requant(pc, 512, ps, 8, 2, 1024, 128, pc, ps, None) == 4
    assert L.agoq_fp8_grad_reduce_requant(pc, 1032, ps, 8, 2, 1024, 128, pc, ps, None) == 5
    torch.cuda.synchronize()
    assert bool((c == 7).all()) and bool((s == 3.0).all())


@pytest.mark.parametrize("as_bf16", [False, True])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("n_groups", [1, 17, 4 * 32 + 3, 30011])
def test_fp8_gradient_accumulate(agoq, ref, group, n_groups, as_bf16):
    n = n_groups * group
    base = wl.grad_host(n, 7100 + n_groups, 1e-4, 0.001, 100.0)
    main_c, main_s = ref.fp8_grad_quant(base, group)
    g32 = wl.grad_host(n, 7200 + n_groups, 1e-4, 0.001, 100.0)
    if n_groups > 8:
        g32[group * 2: group * 3] = 0.0
        main_c[group * 2: group * 3] = 0x80                   # -0 + 0: a dead group with signed zeros
        g32[group * 5: group * 6] = -ref.fp8_grad_dequant(main_c, main_s, group)[group * 5: group * 6]
    if as_bf16:
        t = torch.from_numpy(g32).to(torch.bfloat16)
        g_host = t.view(torch.int16).numpy().view(np.uint16)
        g_dev = t.cuda()
    else:
        g_host, g_dev = g32, torch.from_numpy(g32).cuda()
    want = ref.fp8_grad_accumulate(main_c, main_s, g_host, group)
    d_c, d_s = torch.from_numpy(main_c).cuda(), torch.from_numpy(main_s).cuda()
    out_c, out_s = torch.empty_like(d_c), torch.empty_like(d_s)
    agoq.fp8_grad_accumulate(d_c, d_s, g_dev, group, out_codes=out_c, out_scales=out_s)
    torch.cuda.synchronize()
    assert same_f32(out_s.cpu().numpy(), want[1]) and np.array_equal(out_c.cpu().numpy(), want[0])
    agoq.fp8_grad_accumulate(d_c, d_s, g_dev, group)          # in place
    torch.cuda.synchronize()
    assert same_f32(d_s.cpu().numpy(), want[1]) and np.array_equal(d_c.cpu().numpy(), want[0])
