"""CPU-only checks of the library's host side: it loads, exports every symbol the header
declares, and its pure host helpers give the values the paper prints."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def agoq():
    import paper_2605_00539_amd as lib
    if not os.path.exists(lib.library_path()):
        from paper_2605_00539_amd import build
        build.build()
    lib.load_library()
    return lib


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "agoq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(agoq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(agoq):
    names = declared_symbols()
    assert {"agoq_act_quant", "agoq_act_dequant", "agoq_grad_quant",
            "agoq_grad_reduce_requant"} <= set(names)
    L = ctypes.CDLL(agoq.library_path())
    for name in names:
        assert hasattr(L, name), name


def test_size_helpers(agoq):
    assert agoq.codes_bytes(1 << 20, 4) == 1 << 19
    assert agoq.codes_bytes(1 << 20, 8) == 1 << 20
    assert agoq.codes_bytes(128, 5) == 80 and agoq.codes_bytes(128, 6) == 96
    assert agoq.codes_bytes(128, 7) == -1 and agoq.codes_bytes(128, 3) == -1
    assert agoq.num_groups(4096 * 14336, 128) == 4096 * 14336 // 128
    assert agoq.num_groups(100, 64) == -1
    assert agoq.strerror(0) == "ok" and "group" in agoq.strerror(3)
    assert agoq.version() >= 100


def load_kv(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split(":")
                out[k.strip()] = v.split()
    return out


def test_dbca_values_printed_in_the_paper(agoq):
    gold = load_kv("dbca_four_stages.txt")
    n = int(gold["n_stages"][0])
    assert [agoq.dbca_stored_microbatches(n, i) for i in range(1, n + 1)] == \
        [int(v) for v in gold["stored_microbatches"]]
    assert [agoq.dbca_bits(n, i) for i in range(1, n + 1)] == [int(v) for v in gold["bits"]]
    assert agoq.dbca_stored_microbatches(4, 0) == -1 and agoq.dbca_stored_microbatches(4, 5) == -1
    with pytest.raises(agoq.AgoqError):
        agoq.dbca_bits(4, 5)


def test_dbca_matches_oracle_for_all_small_pipelines(agoq, ref):
    for n in range(1, 33):
        for i in range(1, n + 1):
            assert agoq.dbca_bits(n, i) == ref.dbca_bits(n, i)
            assert agoq.dbca_stored_microbatches(n, i) == ref.dbca_stored_microbatches(n, i)


def test_layer_memory_units_of_the_paper(agoq):
    # Table "memory_comparison": with every stored tensor at 4 bits (code bytes only, ffn = 4h)
    # a layer keeps 0.25U + 0.5U + 2U = 2.75U besides attention's 5U
    gold = {k: float(v[0]) for k, v in load_kv("memory_units.txt").items()}
    tokens, hidden = 4096, 4096
    U = tokens * hidden * 2
    bits = agoq.layer_bitmap(4)
    assert bits == [4, 4, 4, 4, 4]
    stored = agoq.layer_stored_bytes(tokens, hidden, 4 * hidden, 128, bits, with_scales=False)
    want_units = gold["agoq_linear"] + gold["agoq_rmsnorm"] + gold["agoq_act_func"]
    assert stored == int(want_units * U)
    assert want_units + gold["agoq_attention"] == gold["agoq_total"]
    # per component
    one = lambda slot_bits: agoq.layer_stored_bytes(tokens, hidden, 4 * hidden, 128, slot_bits, False)
    assert stored - one([8, 4, 4, 4, 4]) == -int(0.25 * U)       # one norm input: 0.25U at 4 bits
    # scales add 4 bytes per group of 128: 4.25 bits per element in total
    with_scales = agoq.layer_stored_bytes(tokens, hidden, 4 * hidden, 128, bits, True)
    assert with_scales * 16 == stored * 17


def test_stage_bitmaps_average_width(agoq):
    # seq 8192 on the 8B shape: closed forms for the four stage maps (codes + scales)
    want = {4: 178257920, 5: 211812352, 6: 270532608, 8: 346030080}
    for b, total in want.items():
        bits = agoq.layer_bitmap(b)
        assert agoq.layer_stored_bytes(8192, 4096, 14336, 128, bits, True) == total
    assert agoq.layer_bitmap(5) == [8, 4, 8, 4, 4] and agoq.layer_bitmap(6) == [8, 4, 8, 8, 4]
    with pytest.raises(agoq.AgoqError):
        agoq.layer_bitmap(3)
    # native maps: every tensor at the stage's own width, stored bytes scale with it
    for b, stored_b in ((4, 4), (5, 5), (6, 6), (7, 6), (8, 8)):
        bits = agoq.layer_bitmap(b, native=True)
        assert bits == [stored_b] * 5
        codes_only = agoq.layer_stored_bytes(8192, 4096, 14336, 128, bits, False)
        assert codes_only == 8192 * (3 * 4096 + 2 * 14336) * stored_b // 8
    # the paper's budget argument: stage i holds N_i micro-batches at B_i bits; none exceeds stage 1
    n1 = agoq.dbca_stored_microbatches(4, 1)
    for stage in (1, 2, 3, 4):
        b = agoq.layer_bitmap(agoq.dbca_bits(4, stage), native=True)[0]
        ni = agoq.dbca_stored_microbatches(4, stage)
        assert (b - 0.5) * ni <= 4 * n1


def test_generated_isa_has_no_packed_fp32_math(tmp_path):
    """The device code must contain no packed fp32 arithmetic (v_pk_{add,mul,fma}_f32)."""
    import subprocess
    from paper_2605_00539_amd import build
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    text = ""
    for src in build.SOURCES:
        if not src.endswith(".hip"):
            continue
        out = tmp_path / (os.path.basename(src) + ".s")
        subprocess.check_call([build.HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(out), src],
                              stderr=subprocess.DEVNULL)
        text += out.read_text()
    assert "act_quant_kernel" in text and "grad_reduce_kernel" in text and "rmsnorm" in text
    for mnemonic in ("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32"):
        assert mnemonic not in text, mnemonic
    assert "scratch_" not in text                       # no register spills to scratch memory


def test_layer_call_argument_checks(agoq):
    # every rejection happens on the host before anything touches a device, so it can be
    # exercised here with made-up (aligned, never dereferenced) addresses
    import ctypes
    L = agoq.load_library()
    Slot = agoq.ActSlot

    def call(fn, slots, count, group=128):
        arr = (Slot * max(len(slots), 1))(*slots)
        return fn(arr, count, group, None)

    good = Slot(0x10000, 0x20000, 0x30000, 1024, 4)
    for fn in (L.agoq_act_quant_layer, L.agoq_act_dequant_layer):
        assert fn(None, 1, 128, None) == 1
        assert call(fn, [good], 0) == 8
        assert call(fn, [good] * 9, 9) == 8
        assert call(fn, [good], 1, group=32) == 3
        assert call(fn, [good, Slot(0x10000, 0, 0x30000, 1024, 4)], 2) == 1
        assert call(fn, [good, Slot(0x10000, 0x20000, 0x30000, 1024, 7)], 2) == 2
        assert call(fn, [good, Slot(0x10000, 0x20000, 0x30000, 1000, 4)], 2) == 4
        assert call(fn, [good, Slot(0x10000, 0x20000, 0x30000, 0, 4)], 2) == 4
        assert call(fn, [good, Slot(0x10008, 0x20000, 0x30000, 1024, 4)], 2) == 5
    assert "count" in agoq.strerror(8)


def test_profile_summaries_quote_committed_commands():
    """Every summary under profiles/ is short text that quotes the rocprofv3 command that made
    it, and that command runs a committed file (bench.py) and nothing else."""
    import re
    folder = os.path.join(ROOT, "profiles")
    names = sorted(os.listdir(folder))
    assert names, "profiles/ is empty"
    for name in names:
        path = os.path.join(folder, name)
        assert name.endswith((".txt", ".md")), name
        assert os.path.getsize(path) < 64 * 1024, name
        text = open(path).read()
        commands = re.findall(r"rocprofv3 .* -- (\S+) (\S+)", text)
        assert commands, "%s quotes no rocprofv3 command" % name
        for program, script in commands:
            assert program == "python3" and script == "bench.py", (name, program, script)
        # counters and traces never share a run
        for line in text.splitlines():
            if "rocprofv3" in line and "--pmc" in line:
                assert "--kernel-trace" not in line and "--stats" not in line, (name, line)
