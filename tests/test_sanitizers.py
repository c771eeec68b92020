"""AddressSanitizer + UndefinedBehaviorSanitizer pass over the CPU oracle and the library's
host helpers (host code only: no GPU, no HIP runtime).  tests/native/sanitize_check.cpp calls
every oracle entry point and every host helper on exact-size heap buffers -- ragged group
counts, 5- and 6-bit planes, K = 64, strides beyond the extents -- in a build that aborts on
the first finding."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")
def test_oracle_and_host_helpers_under_asan_and_ubsan(tmp_path):
    inc = ["-I", os.path.join(ROOT, "include")]
    ref_o = str(tmp_path / "agoq_ref.o")
    host_o = str(tmp_path / "agoq_host.o")
    drv_o = str(tmp_path / "sanitize_check.o")
    exe = str(tmp_path / "sanitize_check")
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", *SAN, "-c",
                           os.path.join(ROOT, "oracle", "agoq_ref.c"), "-o", ref_o])
    subprocess.check_call(["g++", "-std=c++17", *SAN, *inc, "-c",
                           os.path.join(ROOT, "paper_2605_00539_amd", "csrc", "agoq_host.cpp"), "-o", host_o])
    subprocess.check_call(["g++", "-std=c++17", *SAN, *inc, "-c",
                           os.path.join(ROOT, "tests", "native", "sanitize_check.cpp"), "-o", drv_o])
    # the sanitizer runtimes are linked statically: a preloaded library in the environment
    # would otherwise come before them, which the dynamic runtime refuses
    subprocess.check_call(["g++", *SAN, "-static-libasan", "-static-libubsan", "-fopenmp", drv_o, ref_o, host_o,
                           "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, env=env)
    assert proc.returncode == 0, proc.stdout[-4000:]
    assert "sanitizer run clean" in proc.stdout
    assert "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_the_sanitizer_build_does_catch_an_overrun(tmp_path):
    """The pass above means something only if this build notices a one-byte overrun: a tiny
    program that asks the oracle to write codes into a buffer one byte short must abort."""
    src = tmp_path / "short.c"
    src.write_text(
        "#include <stdint.h>\n#include <stdlib.h>\n"
        "int agoq_ref_act_quant(const uint16_t*, int64_t, int, int, uint8_t*, float*);\n"
        "int main(void) {\n"
        "  uint16_t *x = calloc(128, 2); uint8_t *c = malloc(63); float *s = malloc(4);\n"
        "  x[5] = 0x3F80;\n"
        "  return agoq_ref_act_quant(x, 128, 128, 4, c, s);\n"
        "}\n")
    exe = str(tmp_path / "short")
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", *SAN, "-static-libasan",
                           "-static-libubsan", str(src), os.path.join(ROOT, "oracle", "agoq_ref.c"), "-lm",
                           "-o", exe])
    env = dict(os.environ, OMP_NUM_THREADS="1")
    env.pop("LD_PRELOAD", None)
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120, env=env)
    assert proc.returncode != 0 and "heap-buffer-overflow" in proc.stdout, proc.stdout[-2000:]
