"""The boundary is a C ABI: include/moev.h compiles as strict C99 and C++17, and a plain C program
(no Python, no PyTorch) drives plan -> pack -> drain -> fused conversion on the GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
PKG = os.path.join(ROOT, "paper_2412_15411_amd")


def test_header_is_valid_c_and_cpp(tmp_path):
    src_c = tmp_path / "use.c"
    src_c.write_text('#include "moev.h"\nint main(void) { return sizeof(moev_plan_cfg) > 0 ? 0 : 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", f"-I{INC}", "-c", str(src_c), "-o",
                    str(tmp_path / "c.o")], check=True, capture_output=True, text=True)
    src_cpp = tmp_path / "use.cpp"
    src_cpp.write_text('#include "moev.h"\nint main() { return sizeof(moev_plan_cfg) > 0 ? 0 : 1; }\n')
    subprocess.run(["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", f"-I{INC}", "-c", str(src_cpp), "-o",
                    str(tmp_path / "cpp.o")], check=True, capture_output=True, text=True)


def _build_c_program(tmp_path):
    exe = str(tmp_path / "roundtrip")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", f"-I{INC}", "-I/opt/rocm/include",
           os.path.join(ROOT, "tests", "c_abi", "roundtrip.c"), "-o", exe, f"-L{PKG}", "-l:libmoev.so",
           "-L/opt/rocm/lib", "-lamdhip64", f"-Wl,-rpath,{PKG}", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


def test_c_program_links_against_the_library(tmp_path):
    _build_c_program(tmp_path)


@pytest.mark.gpu
def test_c_program_roundtrip_on_gpu(tmp_path):
    exe = _build_c_program(tmp_path)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stdout + res.stderr
