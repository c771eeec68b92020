"""GPU parity of the one-launch layer calls: every buffer must hold exactly what the oracle
gives for that tensor alone (scales as uint32, code bytes, dequantized bf16 as uint16)."""
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


def make(shapes, seed, dist="normal"):
    return [wl.act_host(rows=r, cols=c, seed=seed + i, dist=dist, outlier_channels=max(1, c // 200),
                        outlier_scale=30.0).reshape(-1) for i, (r, c) in enumerate(shapes)]


def check_layer(agoq, ref, xs_bits, bitmap, group):
    xs = [dev_bf16(x) for x in xs_bits]
    codes, scales = agoq.act_quant_layer(xs, group, bitmap)
    torch.cuda.synchronize()
    want = [ref.act_quant(x, group, b) for x, b in zip(xs_bits, bitmap)]
    for i, ((wc, ws), c, s) in enumerate(zip(want, codes, scales)):
        assert same_f32(s.cpu().numpy(), ws), "scales of tensor %d differ" % i
        assert np.array_equal(c.cpu().numpy(), wc), "codes of tensor %d differ" % i
    outs = agoq.act_dequant_layer(codes, scales, [x.size for x in xs_bits], group, bitmap)
    torch.cuda.synchronize()
    for i, ((wc, ws), x, b, y) in enumerate(zip(want, xs_bits, bitmap, outs)):
        wy = ref.act_dequant(wc, ws, x.size, group, b)
        assert np.array_equal(host_bits(y), wy), "dequantized tensor %d differs" % i


@pytest.mark.parametrize("group", [64, 128])
def test_five_slot_layer_all_stage_maps(agoq, ref, group):
    # the five stored tensors of a small decoder layer (three of width h, two of width ffn),
    # under the mix and the native map of every stage width
    rows, h, ffn = 96, 512, 1408
    xs = make([(rows, h), (rows, h), (rows, h), (rows, ffn), (rows, ffn)], seed=500)
    for b in (4, 5, 6, 8):
        for native in (False, True):
            check_layer(agoq, ref, xs, agoq.layer_bitmap(b, native=native), group)


def test_ragged_sizes_and_every_count(agoq, ref):
    # tensors that end inside a workgroup's tile, in every position, counts 1..8, widths mixed
    sizes = [(1, 128), (3, 640), (257, 384), (40, 4096), (5, 128), (1023, 256), (64, 1152), (9, 8192)]
    widths = [4, 8, 5, 6, 8, 4, 6, 5]
    xs = make(sizes, seed=600, dist="student_t3")
    for count in range(1, 9):
        check_layer(agoq, ref, xs[:count], widths[:count], 128)
    check_layer(agoq, ref, xs[::-1], widths[::-1], 128)


def test_layer_of_the_8b_shape_matches_single_calls(agoq):
    # full 8B-shaped layer (seq 4096): the layer launch against the five single launches
    cfg = wl.CONFIGS["llama8b_act"]
    rows = cfg["acts"]["A"]["rows"]
    h, ffn = cfg["acts"]["A"]["cols"], cfg["acts"]["F"]["cols"]
    bitmap = agoq.layer_bitmap(5)
    xs = []
    for slot in range(5):
        cols = ffn if slot >= 3 else h
        xs.append(wl.act_device(rows, cols, cfg["seed"] + slot, cfg["dist"],
                                wl.n_outlier_channels(cols, cfg["outlier_frac"]),
                                cfg["outlier_scale"]).reshape(-1))
    codes, scales = agoq.act_quant_layer(xs, 128, bitmap)
    outs = agoq.act_dequant_layer(codes, scales, [x.numel() for x in xs], 128, bitmap)
    torch.cuda.synchronize()
    for x, b, c, s, y in zip(xs, bitmap, codes, scales, outs):
        c1, s1 = agoq.act_quant(x, 128, b)
        y1 = agoq.act_dequant(c1, s1, x.numel(), 128, b)
        torch.cuda.synchronize()
        assert torch.equal(c, c1) and torch.equal(s.view(torch.int32), s1.view(torch.int32))
        assert torch.equal(y.view(torch.int16), y1.view(torch.int16))


def test_8b_layer_sampled_against_the_oracle(agoq, ref):
    # the same full-size launch, checked against the oracle on whole rows sampled from each tensor
    cfg = wl.CONFIGS["llama8b_act"]
    rows = cfg["acts"]["A"]["rows"]
    h, ffn = cfg["acts"]["A"]["cols"], cfg["acts"]["F"]["cols"]
    bitmap = agoq.layer_bitmap(6, native=True)
    xs, colsl = [], []
    for slot in range(5):
        cols = ffn if slot >= 3 else h
        colsl.append(cols)
        xs.append(wl.act_device(rows, cols, cfg["seed"] + 10 + slot, cfg["dist"],
                                wl.n_outlier_channels(cols, cfg["outlier_frac"]),
                                cfg["outlier_scale"]).reshape(-1))
    codes, scales = agoq.act_quant_layer(xs, 128, bitmap)
    outs = agoq.act_dequant_layer(codes, scales, [x.numel() for x in xs], 128, bitmap)
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    for x, cols, b, s, y in zip(xs, colsl, bitmap, scales, outs):
        for r in [0, rows - 1] + list(rng.integers(1, rows - 1, 6)):
            xb = host_bits(x[r * cols:(r + 1) * cols])
            wc, ws = ref.act_quant(xb, 128, b)
            wy = ref.act_dequant(wc, ws, cols, 128, b)
            g0 = r * cols // 128
            assert same_f32(s[g0:g0 + cols // 128].cpu().numpy(), ws)
            assert np.array_equal(host_bits(y[r * cols:(r + 1) * cols]), wy)


def test_descriptor_array_can_be_reused_and_freed(agoq, ref):
    xs_bits = make([(8, 256), (16, 128)], seed=700)
    xs = [dev_bf16(x) for x in xs_bits]
    bitmap = [4, 8]
    codes = [torch.zeros(x.numel() * b // 8, dtype=torch.uint8, device="cuda") for x, b in zip(xs, bitmap)]
    scales = [torch.zeros(x.numel() // 128, dtype=torch.float32, device="cuda") for x in xs]
    slots = agoq.layer_slots(xs, bitmap, codes, scales, 128)
    for _ in range(3):
        agoq.act_quant_layer(xs, 128, bitmap, slots=slots)
    torch.cuda.synchronize()
    for x, b, c, s in zip(xs_bits, bitmap, codes, scales):
        wc, ws = ref.act_quant(x, 128, b)
        assert np.array_equal(c.cpu().numpy(), wc) and same_f32(s.cpu().numpy(), ws)


def test_layer_call_in_a_hip_graph(agoq):
    xs_bits = make([(64, 512), (64, 512), (64, 1408)], seed=800)
    xs = [dev_bf16(x) for x in xs_bits]
    bitmap = [8, 4, 6]
    codes, scales = agoq.act_quant_layer(xs, 128, bitmap)
    outs = agoq.act_dequant_layer(codes, scales, [x.numel() for x in xs], 128, bitmap)
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    gc = [torch.zeros_like(c) for c in codes]
    gs = [torch.zeros_like(s) for s in scales]
    go = [torch.zeros_like(o) for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        agoq.act_quant_layer(xs, 128, bitmap, gc, gs)
        agoq.act_dequant_layer(gc, gs, [x.numel() for x in xs], 128, bitmap, outs=go)
    for rep in range(3):
        for o in go:
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for w, o in zip(want, go):
            assert torch.equal(w.view(torch.int16), o.view(torch.int16)), "replay %d" % rep
