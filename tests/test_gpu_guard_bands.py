"""GPU: no call writes outside its output buffers.

Every output is a 16-byte-aligned window inside a larger buffer filled with a canary byte;
after the call the bytes on both sides of every window must still be the canary.  Sizes are
ragged (partial last tiles, tensors smaller than a tile, rows that do not fill their lanes),
which is where a masked store could go wrong.  Parity of the window contents themselves is
the subject of the other GPU tests; here only one cheap property of them is checked (the
scales of a Gaussian tensor are positive)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

CANARY = 0xA5
BAND = 4096          # bytes of canary on each side of a window


@pytest.fixture(scope="module")
def agoq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_00539_amd as lib
    lib.load_library()
    return lib


class Arena:
    """Windows of given byte sizes inside one canary-filled device buffer."""

    def __init__(self, sizes):
        self.offsets = []
        pos = BAND
        for nbytes in sizes:
            self.offsets.append((pos, nbytes))
            pos += (nbytes + 15) // 16 * 16 + BAND
        self.buf = torch.full((pos,), CANARY, dtype=torch.uint8, device="cuda")

    def window(self, i, dtype):
        off, nbytes = self.offsets[i]
        return self.buf[off:off + nbytes].view(dtype)

    def check(self, what):
        host = self.buf.cpu().numpy()
        mask = np.ones(host.size, bool)
        for off, nbytes in self.offsets:
            mask[off:off + nbytes] = False
        bad = np.nonzero(mask & (host != CANARY))[0]
        assert bad.size == 0, "%s wrote outside its outputs, first at byte %d" % (what, int(bad[0]))


def gaussian_bf16(n, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return torch.randn(n, generator=gen, device="cuda").to(torch.bfloat16)


SIZES = [1, 3, 17, 255, 257, 1023, 4097, 8191, 16385, 40001]     # groups


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_activation_calls(agoq, bits, group):
    for n_groups in SIZES:
        n = n_groups * group
        x = gaussian_bf16(n, n_groups)
        a = Arena([n * bits // 8, 4 * n_groups, 2 * n])
        codes, scales, y = a.window(0, torch.uint8), a.window(1, torch.float32), a.window(2, torch.bfloat16)
        agoq.act_quant(x, group, bits, codes=codes, scales=scales)
        agoq.act_dequant(codes, scales, n, group, bits, out=y)
        torch.cuda.synchronize()
        a.check("act_quant/act_dequant bits %d group %d n %d" % (bits, group, n))
        assert bool((scales > 0).all())
        if bits == 4:
            a = Arena([n // 2, 4 * n_groups, 2 * n])
            codes, scales, y = a.window(0, torch.uint8), a.window(1, torch.float32), a.window(2, torch.bfloat16)
            agoq.fp4_act_quant(x, group, codes=codes, scales=scales)
            agoq.fp4_act_dequant(codes, scales, n, group, out=y)
            torch.cuda.synchronize()
            a.check("fp4 calls group %d n %d" % (group, n))


def test_layer_calls(agoq):
    group = 128
    rng = np.random.default_rng(1)
    for trial in range(6):
        count = int(rng.integers(1, 9))
        widths = [int(b) for b in rng.choice([4, 5, 6, 8], count)]
        ns = [group * int(rng.choice(SIZES)) for _ in range(count)]
        xs = [gaussian_bf16(n, 50 + i) for i, n in enumerate(ns)]
        sizes = []
        for n, b in zip(ns, widths):
            sizes += [n * b // 8, 4 * (n // group), 2 * n]
        a = Arena(sizes)
        codes = [a.window(3 * i, torch.uint8) for i in range(count)]
        scales = [a.window(3 * i + 1, torch.float32) for i in range(count)]
        ys = [a.window(3 * i + 2, torch.bfloat16) for i in range(count)]
        agoq.act_quant_layer(xs, group, widths, codes_list=codes, scales_list=scales)
        agoq.act_dequant_layer(codes, scales, ns, group, widths, outs=ys)
        torch.cuda.synchronize()
        a.check("layer calls %s %s" % (widths, ns))


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("fp8", [False, True])
def test_gradient_calls(agoq, fp8, group):
    code_t = torch.uint8 if fp8 else torch.int8
    quant = agoq.fp8_grad_quant if fp8 else agoq.grad_quant
    dequant = agoq.fp8_grad_dequant if fp8 else agoq.grad_dequant
    reduce_ = agoq.fp8_grad_reduce_requant if fp8 else agoq.grad_reduce_requant
    accumulate = agoq.fp8_grad_accumulate if fp8 else agoq.grad_accumulate
    gen = torch.Generator(device="cuda")
    gen.manual_seed(9)
    for n_groups in SIZES:
        n = n_groups * group
        g = torch.randn(n, generator=gen, device="cuda") * 1e-3
        a = Arena([n, 4 * n_groups, 4 * n, n, 4 * n_groups, n, 4 * n_groups])
        codes, scales, f32 = a.window(0, code_t), a.window(1, torch.float32), a.window(2, torch.float32)
        quant(g, group, codes=codes, scales=scales)
        dequant(codes, scales, group, out=f32)
        acc_c, acc_s = a.window(3, code_t), a.window(4, torch.float32)
        accumulate(codes, scales, g, group, out_codes=acc_c, out_scales=acc_s)
        red_c, red_s = a.window(5, code_t), a.window(6, torch.float32)
        for K in (1, 3, 8):
            in_codes = torch.randint(0, 127, (K, n + 48), generator=gen, device="cuda", dtype=torch.int32).to(code_t)
            in_scales = torch.rand((K, n_groups + 4), generator=gen, device="cuda") * 1e-5
            reduce_(in_codes, in_scales, n, group, out_codes=red_c, out_scales=red_s)
        torch.cuda.synchronize()
        a.check("gradient calls fp8 %s group %d n %d" % (fp8, group, n))
        accumulate(codes, scales, g.to(torch.bfloat16), group, out_codes=acc_c, out_scales=acc_s)
        torch.cuda.synchronize()
        a.check("accumulate (bf16 addend) fp8 %s group %d n %d" % (fp8, group, n))


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
@pytest.mark.parametrize("rows,cols", [(1, 128), (7, 640), (33, 5120), (300, 1408), (19, 14336), (3, 16384), (2100, 3584), (2100, 14336)])
def test_fused_calls(agoq, rows, cols, bits):
    import ctypes
    L = agoq.load_library()
    P = ctypes.c_void_p
    group = 128
    n = rows * cols
    x = gaussian_bf16(n, rows + cols).view(rows, cols)
    up = gaussian_bf16(n, rows + cols + 1)
    gamma = torch.ones(cols, dtype=torch.float32, device="cuda")
    st = P(torch.cuda.current_stream().cuda_stream)
    eps = ctypes.c_float(1e-5)
    nb = n * bits // 8
    a = Arena([2 * n, 4 * rows, nb, 4 * (n // group), 2 * n, 4 * rows, 2 * n, nb, 4 * (n // group), nb, 4 * (n // group), 2 * n])
    w = [P(a.buf.data_ptr() + off) for off, _ in a.offsets]
    px, pup, pg = P(x.data_ptr()), P(up.data_ptr()), P(gamma.data_ptr())
    assert L.agoq_rmsnorm_fwd_quant(px, rows, cols, pg, eps, group, bits, w[0], w[1], w[2], w[3], st) == 0
    assert L.agoq_act_dequant_rmsnorm(w[2], w[3], rows, cols, group, bits, pg, eps, w[4], w[5], st) == 0
    assert L.agoq_silu_mul_fwd_quant(px, pup, n, group, bits, bits, w[6], w[7], w[8], w[9], w[10], st) == 0
    assert L.agoq_act_dequant_silu_mul(w[7], w[8], bits, w[9], w[10], bits, n, group, w[11], st) == 0
    torch.cuda.synchronize()
    a.check("fused calls bits %d rows %d cols %d" % (bits, rows, cols))
    assert bool((a.window(1, torch.float32) > 0).all())


def test_binding_refuses_buffers_that_are_too_small(agoq):
    """The C ABI takes plain pointers; the binding still knows the sizes and checks them."""
    group, n = 128, 128 * 64
    x = gaussian_bf16(n, 1)
    g = torch.zeros(n, dtype=torch.float32, device="cuda")
    ok_codes = torch.empty(n, dtype=torch.uint8, device="cuda")
    ok_scales = torch.empty(n // group, dtype=torch.float32, device="cuda")
    small_codes = torch.empty(n // 2 - 16, dtype=torch.uint8, device="cuda")
    small_scales = torch.empty(n // group - 1, dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        agoq.act_quant(x, group, 4, codes=small_codes, scales=ok_scales)
    with pytest.raises(ValueError):
        agoq.act_quant(x, group, 4, codes=ok_codes, scales=small_scales)
    with pytest.raises(ValueError):
        agoq.act_dequant(small_codes, ok_scales, n, group, 4)
    with pytest.raises(ValueError):
        agoq.act_dequant(ok_codes, ok_scales, n, group, 8, out=torch.empty(n - 8, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(ValueError):
        agoq.act_quant_layer([x, x], group, [4, 8], codes_list=[ok_codes, small_codes], scales_list=[ok_scales, ok_scales])
    with pytest.raises(ValueError):
        agoq.grad_quant(g, group, codes=ok_codes.view(torch.int8)[: n - 16], scales=ok_scales)
    with pytest.raises(ValueError):
        agoq.grad_dequant(ok_codes.view(torch.int8), small_scales, group)
    with pytest.raises(ValueError):
        agoq.grad_reduce_requant(torch.zeros((2, n), dtype=torch.int8, device="cuda"),
                                 torch.zeros((2, n // group), dtype=torch.float32, device="cuda"), n, group,
                                 out_scales=small_scales)
    with pytest.raises(ValueError):
        agoq.grad_accumulate(ok_codes.view(torch.int8), small_scales, g, group)
    with pytest.raises(ValueError):
        agoq.act_dequant_rmsnorm(small_codes, ok_scales, 64, 128, group, 4,
                                 torch.ones(128, dtype=torch.float32, device="cuda"), 1e-5)
    with pytest.raises(ValueError):
        agoq.act_dequant_silu_mul(ok_codes, ok_scales, 4, small_codes, ok_scales, 4, n, group)
    torch.cuda.synchronize()
