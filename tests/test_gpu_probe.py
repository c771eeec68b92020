"""GPU: the measurement-aid copy kernel (agoq_probe_stream) moves exactly the bytes it is said
to move -- the floor figures of the benchmark rest on that -- and rejects bad arguments."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
P = ctypes.c_void_p


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2605_00539_amd as lib
    return lib.load_library()


def expected(src_words, load, store, items):
    """What the kernel writes: every item folds its loaded words with xor and stores the
    result widened to the store width as {w, ~w, w + 1, w - 1}[: store / 4]."""
    w = src_words[: items * (load // 4)].reshape(items, load // 4)
    f = np.bitwise_xor.reduce(w, axis=1).astype(np.uint32)
    cols = [f, ~f, f + np.uint32(1), f - np.uint32(1)][: store // 4]
    return np.stack(cols, axis=1).reshape(-1)


@pytest.mark.parametrize("load", [4, 8, 16])
@pytest.mark.parametrize("store", [4, 8, 16])
@pytest.mark.parametrize("items", [1, 511, 512, 513, 3 * 512 * 256 + 77])
def test_probe_moves_the_stated_bytes(L, load, store, items):
    rng = np.random.default_rng(items + load + store)
    src_h = rng.integers(0, 2**32, size=items * (load // 4) + 8, dtype=np.uint32)
    src = torch.from_numpy(src_h.view(np.int32)).cuda()
    guard = 64
    dst = torch.full((items * (store // 4) + guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    st = P(torch.cuda.current_stream().cuda_stream)
    assert L.agoq_probe_stream(P(src.data_ptr()), load, P(dst.data_ptr()), store, items, st) == 0
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint32)
    assert np.array_equal(got[: items * (store // 4)], expected(src_h, load, store, items))
    assert np.all(got[items * (store // 4):] == 0x5A5A5A5A), "wrote past the last item"


def test_probe_read_only_form_writes_nothing(L):
    items = 100000
    src = torch.randint(0, 255, (items * 16,), dtype=torch.uint8, device="cuda")
    dst = torch.full((1024,), 7, dtype=torch.int32, device="cuda")
    st = P(torch.cuda.current_stream().cuda_stream)
    for load in (4, 8, 16):
        assert L.agoq_probe_stream(P(src.data_ptr()), load, P(dst.data_ptr()), 0, items, st) == 0
    torch.cuda.synchronize()
    assert bool((dst == 7).all())


def test_probe_error_codes(L):
    buf = torch.zeros(4096, dtype=torch.int32, device="cuda")
    st = P(torch.cuda.current_stream().cuda_stream)
    p = buf.data_ptr()
    assert L.agoq_probe_stream(None, 16, P(p), 16, 16, st) == 1
    assert L.agoq_probe_stream(P(p), 16, None, 16, 16, st) == 1
    assert L.agoq_probe_stream(P(p), 12, P(p + 8192), 16, 16, st) == 2
    assert L.agoq_probe_stream(P(p), 16, P(p + 8192), 2, 16, st) == 2
    assert L.agoq_probe_stream(P(p), 16, P(p + 8192), 16, 0, st) == 4
    assert L.agoq_probe_stream(P(p), 16, P(p + 8192), 16, -5, st) == 4
    assert L.agoq_probe_stream(P(p + 4), 16, P(p + 8192), 16, 16, st) == 5
    assert L.agoq_probe_stream(P(p), 16, P(p + 8196), 16, 16, st) == 5
    torch.cuda.synchronize()
    assert not bool(buf.any()), "a rejected call launched something"
