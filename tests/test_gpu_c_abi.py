"""The C ABI used from a plain C99 program (tests/c/tc_example.c), with no Python
and no PyTorch in the process: the library must stand on the HIP runtime alone."""

import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BIN = os.path.join(ROOT, "tests", "c", "tc_example.bin")


def test_header_is_valid_c99_and_cxx(tmp_path):
    # CPU-only: include/tc.h on its own compiles as C99 and as C++17
    for lang, std, comp in (("c", "c99", "gcc"), ("c++", "c++17", "g++")):
        src = os.path.join(str(tmp_path), "t." + ("c" if lang == "c" else "cpp"))
        with open(src, "w") as f:
            f.write('#include "tc.h"\nint main(void) { tc_stats s; (void)s; return TC_OK; }\n')
        subprocess.check_call([comp, "-std=" + std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                               "-I", os.path.join(ROOT, "include"), src])


@pytest.mark.gpu
def test_worked_example_from_plain_c():
    assert os.path.exists(BIN), "tests/c/tc_example.bin is missing: run `python -m paper_2511_14124_amd.build` first"
    p = subprocess.run([BIN], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0 and "tc_example: ok" in p.stdout, p.stdout + p.stderr


@pytest.mark.gpu
def test_optimizer_state_example_from_plain_c():
    # the two-tier mode (host cache over a file) through the same header, the update done by the C program itself
    exe = os.path.join(ROOT, "tests", "c", "tc_opt_example.bin")
    assert os.path.exists(exe), "tests/c/tc_opt_example.bin is missing: run `python -m paper_2511_14124_amd.build` first"
    p = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0 and "tc_opt_example: ok" in p.stdout, p.stdout + p.stderr
