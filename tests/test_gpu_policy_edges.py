"""GPU parity at the sizes where the library switches launch shape (vectors per lane, paced
stores, occupancy cap), each with a ragged last tile: the result must not depend on the shape
chosen.  Bit for bit against the oracle."""
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


def compute_units():
    return torch.cuda.get_device_properties(0).multi_processor_count


@pytest.mark.parametrize("bits", [4, 5, 8])
def test_dequant_around_the_resident_grid_thresholds(agoq, ref, bits):
    # one round of 512-lane workgroups with four vectors per lane, and one and a half
    cus = compute_units()
    one_round = cus * 4 * 512 * 4 * 8            # elements
    for numel in (one_round - 128, one_round, one_round + 128, one_round * 3 // 2 - 128,
                  one_round * 3 // 2 + 128):
        x = wl.act_device(numel // 128, 128, 900 + bits, "normal", 2, 30.0).reshape(-1)
        xb = host_bits(x)
        wc, ws = ref.act_quant(xb, 128, bits)
        wy = ref.act_dequant(wc, ws, numel, 128, bits)
        codes, scales = agoq.act_quant(x, 128, bits)
        y = agoq.act_dequant(codes, scales, numel, 128, bits)
        torch.cuda.synchronize()
        assert np.array_equal(codes.cpu().numpy(), wc), (numel, "codes")
        assert same_f32(scales.cpu().numpy(), ws), (numel, "scales")
        assert np.array_equal(host_bits(y), wy), (numel, "dequantized")
        del x, codes, scales, y


@pytest.mark.parametrize("K", [4, 5, 6, 7, 8, 12, 16])
@pytest.mark.parametrize("group", [64, 128])
def test_reduce_around_the_two_vector_threshold(agoq, ref, K, group):
    # from 2,500,000 vectors of 16 elements on, the reduce takes two vectors per lane in a kernel
    # compiled for the chunk count (K = 5, 6, 7, 8, 12, 16; K = 4 stays on the run-time-K kernel)
    edge = 2500000 * 16 // 2048 * 2048           # elements, rounded to whole groups
    rng = np.random.default_rng(1000 + K)
    sizes = (edge - group, edge + 37 * group) if K >= 12 else (edge - group, edge, edge + group, edge + 37 * group)
    for numel in sizes:
        stride_c = numel + 16 * int(rng.integers(0, 5))
        stride_s = numel // group + int(rng.integers(0, 7))
        codes = rng.integers(-127, 128, size=(K, stride_c), dtype=np.int8)
        scales = (rng.random((K, stride_s), dtype=np.float32) * 1e-3 + 1e-6).astype(np.float32)
        scales[:, ::97] = 0.0                     # dead groups among live ones
        wc, ws = ref.grad_reduce_requant(codes, scales, numel, group)
        dc = torch.from_numpy(codes).cuda()
        ds = torch.from_numpy(scales).cuda()
        oc, osc = agoq.grad_reduce_requant(dc, ds, numel, group)
        torch.cuda.synchronize()
        assert np.array_equal(oc.cpu().numpy(), wc), (numel, "codes")
        assert same_f32(osc.cpu().numpy(), ws), (numel, "scales")
        del dc, ds, oc, osc


@pytest.mark.parametrize("group", [64, 128])
def test_stochastic_reduce_around_the_two_vector_threshold(agoq, ref, group):
    # K = 8 is the one chunk count whose compile-time shapes (one and two vectors per lane) also
    # exist for stochastic rounding: both sides of the size threshold, and K = 7 (run-time K)
    edge = 2500000 * 16 // 2048 * 2048
    rng = np.random.default_rng(77 + group)
    for K, numel in ((8, edge - group), (8, edge + 37 * group), (7, edge + 37 * group)):
        stride_c = numel + 32
        stride_s = numel // group + 3
        codes = rng.integers(-127, 128, size=(K, stride_c), dtype=np.int8)
        scales = (rng.random((K, stride_s), dtype=np.float32) * 1e-3 + 1e-6).astype(np.float32)
        scales[:, ::97] = 0.0
        seed = 0xABCD0000 + K
        wc, ws = ref.grad_reduce_requant_sr(codes, scales, numel, group, seed)
        dc = torch.from_numpy(codes).cuda()
        ds = torch.from_numpy(scales).cuda()
        oc, osc = agoq.grad_reduce_requant(dc, ds, numel, group, sr_seed=seed)
        torch.cuda.synchronize()
        assert np.array_equal(oc.cpu().numpy(), wc), (K, numel, "codes")
        assert same_f32(osc.cpu().numpy(), ws), (K, numel, "scales")
        del dc, ds, oc, osc
