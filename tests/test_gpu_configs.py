"""GPU parity at the full sizes of the benchmark configurations, through the same entry
points and launch shapes that bench.py times.  Inputs come from the seeded device
generators (the recipe of workloads.py); every output element is compared with the oracle.
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


def bits_of(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def eq_f32(dev_t, host):
    return np.array_equal(dev_t.cpu().numpy().view(np.uint32), host.view(np.uint32))


def check_act_full(agoq, ref, x, group, bits):
    """x: bf16 device tensor.  Quantize + dequantize on both sides, compare everything."""
    flat = x.reshape(-1)
    n = flat.numel()
    codes, scales = agoq.act_quant(flat, group, bits)
    y = agoq.act_dequant(codes, scales, n, group, bits)
    torch.cuda.synchronize()
    xb = bits_of(flat)
    oc, os_ = ref.act_quant(xb, group, bits)
    assert eq_f32(scales, os_), "scales differ"
    assert np.array_equal(codes.cpu().numpy(), oc), "codes differ"
    oy = ref.act_dequant(oc, os_, n, group, bits)
    assert np.array_equal(bits_of(y), oy), "dequantized values differ"
    # property that holds at any size: every live group carries a code of magnitude qmax
    qmax = (1 << (bits - 1)) - 1
    live = os_ > 0
    if bits == 8:
        mags = np.abs(oc.view(np.int8).astype(np.int16)).reshape(-1, group).max(axis=1)
        assert np.all(mags[live] == qmax)


def act_tensor(cfg, rows, cols, seed):
    return wl.act_device(rows, cols, seed, cfg["dist"],
                         wl.n_outlier_channels(cols, cfg["outlier_frac"]), cfg["outlier_scale"])


# ---- config 2: LLaMA-8B-shaped activations, seq 4096 --------------------------------

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("name", ["A", "F"])
def test_llama8b_activations(agoq, ref, name, bits):
    cfg = wl.CONFIGS["llama8b_act"]
    shape = cfg["acts"][name]
    x = act_tensor(cfg, shape["rows"], shape["cols"], cfg["seed"] + (0 if name == "A" else 3))
    check_act_full(agoq, ref, x, cfg["group"], bits)


# ---- config 4: 32B-shaped activations, heavy tails, both group sizes ----------------

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("name", ["A", "F"])
def test_llama32b_activations(agoq, ref, name, group, bits):
    cfg = wl.CONFIGS["llama32b_act"]
    shape = cfg["acts"][name]
    x = act_tensor(cfg, shape["rows"], shape["cols"], cfg["seed"] + (0 if name == "A" else 1))
    check_act_full(agoq, ref, x, group, bits)


# ---- config 5: a full layer at seq 8192 under the four stage bit maps ---------------

def test_stage_sweep_layer_activations(agoq, ref):
    cfg = wl.CONFIGS["stage_sweep"]
    rows, hidden, ffn, group = cfg["rows"], cfg["hidden"], cfg["ffn"], cfg["group"]
    shapes = [hidden, hidden, hidden, ffn, ffn]          # norm1-in, oproj-in, norm2-in, gate, up
    maps = {b: agoq.layer_bitmap(b) for b in (agoq.dbca_bits(4, s) for s in (1, 2, 3, 4))}
    native = {b: agoq.layer_bitmap(b, native=True) for b in maps}
    assert sorted(maps) == [4, 5, 6, 8]
    for slot, cols in enumerate(shapes):
        x = act_tensor(cfg, rows, cols, cfg["seed"] + slot)
        for bits in sorted({m[slot] for m in maps.values()} | {m[slot] for m in native.values()}):
            check_act_full(agoq, ref, x, group, bits)
        del x
    # bytes saved against bf16, closed form (codes + scales)
    bf16_bytes = rows * (3 * hidden + 2 * ffn) * 2
    stored = {b: agoq.layer_stored_bytes(rows, hidden, ffn, group, m, True) for b, m in maps.items()}
    assert bf16_bytes == 671088640
    assert stored == {4: 178257920, 5: 211812352, 6: 270532608, 8: 346030080}
    stored_native = {b: agoq.layer_stored_bytes(rows, hidden, ffn, group, m, True) for b, m in native.items()}
    assert stored_native == {b: bf16_bytes // 16 * b + 4 * (bf16_bytes // 2 // group) for b in (4, 5, 6, 8)}


# ---- configs 3 and 5: one decoder layer's gradients, K = 8 and K = 16 ----------------

def quantized_peers(ref, cfg_grad, seeds, group):
    """K seeded gradients generated on the device, quantized by the ORACLE on the host."""
    codes, scales = [], []
    for seed in seeds:
        g = wl.grad_device(cfg_grad["n"], seed, cfg_grad["sigma"], cfg_grad["spike_frac"],
                           cfg_grad["spike_scale"])
        c, s = ref.grad_quant(g.cpu().numpy(), group)
        codes.append(c)
        scales.append(s)
        del g
    return np.stack(codes), np.stack(scales)


def test_llama8b_gradient_store(agoq, ref):
    cfg = wl.CONFIGS["llama8b_grad"]
    g = wl.grad_device(cfg["n"], cfg["seed"], cfg["sigma"], cfg["spike_frac"], cfg["spike_scale"])
    codes, scales = agoq.grad_quant(g, cfg["group"])
    torch.cuda.synchronize()
    oc, os_ = ref.grad_quant(g.cpu().numpy(), cfg["group"])
    assert eq_f32(scales, os_)
    assert np.array_equal(codes.cpu().numpy(), oc)
    # int8 + scales against fp32: the paper's "gradient memory by 75%"
    assert codes.numel() + 4 * scales.numel() == 224919552
    assert g.numel() * 4 == 872415232


@pytest.mark.parametrize("config,K", [("llama8b_grad", 8), ("stage_sweep", 16)])
def test_gradient_reduce_full_and_share(agoq, ref, config, K):
    cfg = wl.CONFIGS[config]
    gcfg = cfg if config == "llama8b_grad" else cfg["grad"]
    group = cfg["group"]
    n = gcfg["n"]
    assert cfg["K"] == K
    in_codes, in_scales = quantized_peers(ref, gcfg, [cfg["seed"] + 1 + k for k in range(K)], group)
    d_codes = torch.from_numpy(in_codes).cuda()
    d_scales = torch.from_numpy(in_scales).cuda()
    # headline: every chunk is a whole layer gradient
    got_c, got_s = agoq.grad_reduce_requant(d_codes, d_scales, n, group)
    torch.cuda.synchronize()
    want_c, want_s = ref.grad_reduce_requant(in_codes, in_scales, n, group)
    assert eq_f32(got_s, want_s)
    assert np.array_equal(got_c.cpu().numpy(), want_c)
    assert np.all(np.abs(want_c.reshape(-1, group).astype(np.int16)).max(axis=1)[want_s > 0] == 127)
    # share variant: this GPU's 1/K shard of the layer, chunk stride = the full length
    ns = n // K
    assert ns % group == 0
    for shard in (0, K - 1):
        off = shard * ns
        sub_c = d_codes[:, off:]
        sub_s = d_scales[:, off // group:]
        out_c = torch.empty(ns, dtype=torch.int8, device="cuda")
        out_s = torch.empty(ns // group, dtype=torch.float32, device="cuda")
        L = agoq.load_library()
        import ctypes
        P = ctypes.c_void_p
        rc = L.agoq_grad_reduce_requant(P(sub_c.data_ptr()), n, P(sub_s.data_ptr()), n // group, K,
                                        ns, group, P(out_c.data_ptr()), P(out_s.data_ptr()),
                                        P(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()
        assert np.array_equal(out_c.cpu().numpy(), want_c[off:off + ns])
        assert eq_f32(out_s, want_s[off // group:(off + ns) // group])
