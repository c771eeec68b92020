"""GPU parity of the stochastic-rounding variant: the library's *_sr calls against the oracle's,
bit for bit, on the same seeded inputs and the same seeds (the hash is reproduced on both
sides; nothing random happens at run time)."""
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


def host_bits(t_bf16):
    return t_bf16.view(torch.int16).cpu().numpy().view(np.uint16)


def same_f32(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_act_quant_sr_matches_oracle(agoq, ref, bits, group):
    # several tiles and a ragged tail, outlier channels, a dead group, a non-finite group
    rows, cols = 301, 1024 + group
    x = wl.act_device(rows, cols, 4000 + bits, "normal", 6, 30.0).reshape(-1).clone()
    x[5 * group:6 * group] = 0
    x[9 * group + 3] = float("inf")
    xb = host_bits(x)
    for seed in (0, 1, 0xFFFFFFFF, 20260517):
        want = ref.act_quant_sr(xb, group, bits, seed)
        got = agoq.act_quant(x, group, bits, sr_seed=seed)
        torch.cuda.synchronize()
        assert np.array_equal(got[0].cpu().numpy(), want[0]), (seed, "codes")
        assert same_f32(got[1].cpu().numpy()[:5], want[1][:5]) and np.array_equal(
            got[1].cpu().numpy().view(np.uint32), want[1].view(np.uint32)), (seed, "scales")
    # a different seed gives different codes, the nearest-rounding call yet others
    a = agoq.act_quant(x, group, bits, sr_seed=7)[0]
    b = agoq.act_quant(x, group, bits, sr_seed=8)[0]
    c = agoq.act_quant(x, group, bits)[0]
    assert not torch.equal(a, b) and not torch.equal(a, c)
    # the stored tensor decodes with the ordinary dequantize
    y = agoq.act_dequant(a, agoq.act_quant(x, group, bits, sr_seed=7)[1], x.numel(), group, bits)
    wy = ref.act_dequant(*ref.act_quant_sr(xb, group, bits, 7), x.numel(), group, bits)
    nan = np.isnan(wl_f32(wy))
    assert np.array_equal(host_bits(y)[~nan], wy[~nan])


def wl_f32(bits16):
    return (bits16.astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("group", [64, 128])
def test_grad_quant_sr_matches_oracle(agoq, ref, group):
    n = group * 4099
    g = wl.grad_host(n, 77, 1e-4, 0.001, 100.0)
    g[3 * group:4 * group] = 0.0
    for seed in (3, 0x80000000):
        want = ref.grad_quant_sr(g, group, seed)
        got = agoq.grad_quant(torch.from_numpy(g).cuda(), group, sr_seed=seed)
        torch.cuda.synchronize()
        assert np.array_equal(got[0].cpu().numpy(), want[0]) and same_f32(got[1].cpu().numpy(), want[1])


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 12, 16, 17])
def test_reduce_requant_sr_matches_oracle(agoq, ref, K, group):
    rng = np.random.default_rng(6000 + K)
    n_groups = 2 * 512 * 16 // group + 5          # two blocks and a ragged tail
    n = n_groups * group
    stride_c, stride_s = n + 48, n_groups + 2
    in_codes = rng.integers(-127, 128, size=(K, stride_c)).astype(np.int8)
    in_scales = (rng.random((K, stride_s)) * 1e-5 + 1e-9).astype(np.float32)
    in_scales[:, 2] = 0.0
    seed = 900 + K
    want = ref.grad_reduce_requant_sr(in_codes, in_scales, n, group, seed)
    got = agoq.grad_reduce_requant(torch.from_numpy(in_codes).cuda(), torch.from_numpy(in_scales).cuda(), n,
                                   group, sr_seed=seed)
    torch.cuda.synchronize()
    assert same_f32(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[0].cpu().numpy(), want[0])


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("addend", ["f32", "bf16"])
def test_grad_accumulate_sr_matches_oracle_and_is_unbiased(agoq, ref, addend, group):
    n = group * 2053
    base = wl.grad_host(n, 88, 1e-4, 0.001, 100.0)
    main_c, main_s = ref.grad_quant(base, group)
    new = wl.grad_host(n, 89, 3e-5)
    if addend == "bf16":
        new_t = torch.from_numpy(new).to(torch.bfloat16)
        new_h = new_t.view(torch.int16).numpy().view(np.uint16)
        new_d = new_t.cuda()
    else:
        new_h, new_d = new, torch.from_numpy(new).cuda()
    mc, ms = torch.from_numpy(main_c).cuda(), torch.from_numpy(main_s).cuda()
    for seed in (11, 12):
        want = ref.grad_accumulate_sr(main_c, main_s, new_h, group, seed)
        oc, osc = torch.empty_like(mc), torch.empty_like(ms)
        agoq.grad_accumulate(mc, ms, new_d, group, out_codes=oc, out_scales=osc, sr_seed=seed)
        torch.cuda.synchronize()
        assert np.array_equal(oc.cpu().numpy(), want[0]) and same_f32(osc.cpu().numpy(), want[1])
    # in place
    ic, isc = mc.clone(), ms.clone()
    agoq.grad_accumulate(ic, isc, new_d, group, sr_seed=11)
    torch.cuda.synchronize()
    want = ref.grad_accumulate_sr(main_c, main_s, new_h, group, 11)
    assert np.array_equal(ic.cpu().numpy(), want[0]) and same_f32(isc.cpu().numpy(), want[1])


def test_full_size_gradient_store_sr(agoq, ref):
    cfg = wl.CONFIGS["llama8b_grad"]
    n = cfg["n"] // 8                             # the per-GPU shard: 27,262,976 elements
    g = wl.grad_device(n, cfg["seed"] + 5, cfg["sigma"], cfg["spike_frac"], cfg["spike_scale"])
    got = agoq.grad_quant(g, cfg["group"], sr_seed=424242)
    torch.cuda.synchronize()
    want = ref.grad_quant_sr(g.cpu().numpy(), cfg["group"], 424242)
    assert np.array_equal(got[0].cpu().numpy(), want[0]) and same_f32(got[1].cpu().numpy(), want[1])
    # unbiased where nearest rounding is not: mean error over the tensor, in units of the scale
    s = np.repeat(want[1], cfg["group"]).astype(np.float64)
    live = s > 0
    x = g.cpu().numpy().astype(np.float64)
    err_sr = ((want[0].astype(np.float64) * s - x)[live] / s[live])
    assert abs(err_sr.mean() + 1 / 512) < 5 * err_sr.std() / np.sqrt(err_sr.size) + 1e-4
