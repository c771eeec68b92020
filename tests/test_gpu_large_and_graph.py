"""GPU: sizes beyond 2^32 elements (64-bit indexing), and capture of the path in a HIP graph.

At these sizes the oracle checks sampled groups one by one: groups are independent, so the
inputs of a set of groups (first, last, around every 2^31 / 2^32 element boundary, and random
ones) are gathered, quantized by the oracle as a small tensor, and compared with the same
groups of the GPU output.
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


def sample_groups(n_groups, group, boundaries, rng, extra=4000):
    picks = {0, 1, n_groups - 2, n_groups - 1}
    for b in boundaries:
        g = b // group
        for d in range(-3, 4):
            if 0 <= g + d < n_groups:
                picks.add(g + d)
    picks.update(int(v) for v in rng.integers(0, n_groups, extra))
    return np.array(sorted(picks), np.int64)


def test_activation_beyond_2_to_32_elements(agoq, ref):
    group, bits = 128, 4
    n = (1 << 32) + 128 * 1031                     # 8.6 GB of bf16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    x = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    chunk = 1 << 28
    for off in range(0, n, chunk):                 # fill in pieces: no 17 GB fp32 temporary
        m = min(chunk, n - off)
        x[off:off + m] = torch.randn(m, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    codes, scales = agoq.act_quant(x, group, bits)
    y = agoq.act_dequant(codes, scales, n, group, bits)
    torch.cuda.synchronize()
    n_groups = n // group
    rng = np.random.default_rng(5)
    gs = sample_groups(n_groups, group, [1 << 31, 1 << 32, (1 << 32) + (1 << 31) // 64], rng)
    idx = torch.from_numpy(gs).cuda()
    xs = x.view(n_groups, group)[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    oc, os_ = ref.act_quant(xs, group, bits)
    got_c = codes.view(n_groups, group * bits // 8)[idx].cpu().numpy().reshape(-1)
    got_s = scales[idx].cpu().numpy()
    assert np.array_equal(got_s.view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(got_c, oc)
    oy = ref.act_dequant(oc, os_, xs.size, group, bits)
    got_y = y.view(n_groups, group)[idx].view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)
    assert np.array_equal(got_y, oy)
    # properties over the whole tensor: no dead groups in Gaussian data, every group is full scale
    assert bool((scales > 0).all())


def test_reduce_beyond_2_to_31_elements(agoq, ref):
    group, K = 128, 2
    n = (1 << 31) + 128 * 4099                     # chunk offsets pass 2^31 and 2^32 bytes
    gen = torch.Generator(device="cuda")
    gen.manual_seed(78)
    in_codes = torch.randint(-127, 128, (K, n), generator=gen, device="cuda", dtype=torch.int8)
    in_scales = torch.rand((K, n // group), generator=gen, device="cuda", dtype=torch.float32) * 1e-5
    out_c, out_s = agoq.grad_reduce_requant(in_codes, in_scales, n, group)
    torch.cuda.synchronize()
    n_groups = n // group
    rng = np.random.default_rng(6)
    gs = sample_groups(n_groups, group, [1 << 31, (1 << 31) - (1 << 20)], rng)
    idx = torch.from_numpy(gs).cuda()
    sc = in_codes.view(K, n_groups, group)[:, idx].reshape(K, -1).cpu().numpy()
    ss = in_scales[:, idx].cpu().numpy()
    want_c, want_s = ref.grad_reduce_requant(np.ascontiguousarray(sc), np.ascontiguousarray(ss),
                                             gs.size * group, group)
    assert np.array_equal(out_s[idx].cpu().numpy().view(np.uint32), want_s.view(np.uint32))
    assert np.array_equal(out_c.view(n_groups, group)[idx].cpu().numpy().reshape(-1), want_c)
    # gradient store and local accumulation on the same large index range
    g = torch.empty(n, dtype=torch.float32, device="cuda")
    g.normal_(0.0, 1e-4, generator=gen)
    qc, qs = agoq.grad_quant(g, group)
    agoq.grad_accumulate(out_c, out_s, g, group)          # in place on the reduced gradient
    torch.cuda.synchronize()
    gh = g.view(n_groups, group)[idx].cpu().numpy().reshape(-1)
    wc, ws = ref.grad_quant(gh, group)
    assert np.array_equal(qs[idx].cpu().numpy().view(np.uint32), ws.view(np.uint32))
    assert np.array_equal(qc.view(n_groups, group)[idx].cpu().numpy().reshape(-1), wc)
    ac, as_ = ref.grad_accumulate(want_c, want_s, gh, group)
    assert np.array_equal(out_s[idx].cpu().numpy().view(np.uint32), as_.view(np.uint32))
    assert np.array_equal(out_c.view(n_groups, group)[idx].cpu().numpy().reshape(-1), ac)


def test_step_captured_in_a_hip_graph(agoq, ref):
    """The library neither allocates nor synchronizes, so a caller may capture it.  Replays
    with fresh inputs (eager work and synchronizations in between) must each match the oracle."""
    group = 128
    rows, cols = 512, 4096
    n = rows * cols
    ng = 128 * 8192
    K = 4
    x = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    g = torch.zeros(ng, dtype=torch.float32, device="cuda")
    in_codes = torch.zeros((K, ng), dtype=torch.int8, device="cuda")
    in_scales = torch.zeros((K, ng // group), dtype=torch.float32, device="cuda")
    c4 = torch.empty(n // 2, dtype=torch.uint8, device="cuda")
    c6 = torch.empty(n * 6 // 8, dtype=torch.uint8, device="cuda")
    s4 = torch.empty(n // group, dtype=torch.float32, device="cuda")
    s6 = torch.empty(n // group, dtype=torch.float32, device="cuda")
    y4 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    y6 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    gc = torch.empty(ng, dtype=torch.int8, device="cuda")
    gs = torch.empty(ng // group, dtype=torch.float32, device="cuda")
    rc = torch.empty(ng, dtype=torch.int8, device="cuda")
    rs = torch.empty(ng // group, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def step():
        agoq.act_quant(x, group, 4, codes=c4, scales=s4)
        agoq.act_quant(x, group, 6, codes=c6, scales=s6)
        agoq.grad_quant(g, group, codes=gc, scales=gs)
        agoq.grad_reduce_requant(in_codes, in_scales, ng, group, out_codes=rc, out_scales=rs)
        agoq.grad_accumulate(rc, rs, g, group)
        agoq.act_dequant(c4, s4, n, group, 4, out=y4)
        agoq.act_dequant(c6, s6, n, group, 6, out=y6)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                         # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        xh = wl.act_host(rows, cols, 900 + rep, outlier_channels=20, outlier_scale=30.0).reshape(-1)
        gh = wl.grad_host(ng, 910 + rep, 1e-4, 0.001, 100.0)
        pairs = [ref.grad_quant(wl.grad_host(ng, 920 + 10 * rep + k, 1e-4, 0.001, 100.0), group) for k in range(K)]
        x.copy_(torch.from_numpy(xh.view(np.int16)).cuda().view(torch.bfloat16))
        g.copy_(torch.from_numpy(gh).cuda())
        in_codes.copy_(torch.from_numpy(np.stack([p[0] for p in pairs])).cuda())
        in_scales.copy_(torch.from_numpy(np.stack([p[1] for p in pairs])).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for bits, c, s, y in ((4, c4, s4, y4), (6, c6, s6, y6)):
            oc, os_ = ref.act_quant(xh, group, bits)
            assert np.array_equal(c.cpu().numpy(), oc) and np.array_equal(s.cpu().numpy().view(np.uint32), os_.view(np.uint32))
            assert np.array_equal(y.view(torch.int16).cpu().numpy().view(np.uint16), ref.act_dequant(oc, os_, n, group, bits))
        wc, ws = ref.grad_quant(gh, group)
        assert np.array_equal(gc.cpu().numpy(), wc) and np.array_equal(gs.cpu().numpy().view(np.uint32), ws.view(np.uint32))
        r_c, r_s = ref.grad_reduce_requant(np.stack([p[0] for p in pairs]), np.stack([p[1] for p in pairs]), ng, group)
        a_c, a_s = ref.grad_accumulate(r_c, r_s, gh, group)
        assert np.array_equal(rc.cpu().numpy(), a_c) and np.array_equal(rs.cpu().numpy().view(np.uint32), a_s.view(np.uint32))


def test_c_abi_from_a_torch_free_client():
    """tests/native/cabi_check (built by __graft_entry__.build()) drives the library with
    hipMalloc'd memory and compares with the oracle it links; no Python, no torch in that process."""
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    exe = os.path.join(here, "native", "cabi_check")
    if not os.path.exists(exe):
        import sys
        sys.path.insert(0, os.path.dirname(here))
        import __graft_entry__
        exe = __graft_entry__.build_native_check()
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert proc.returncode == 0, proc.stdout
    assert "all C-ABI checks passed" in proc.stdout
    assert proc.stdout.count("match") == 12 and "MISMATCH" not in proc.stdout
