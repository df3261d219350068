"""The public header is plain C: it compiles under strict C99 and under C++, and a C program
linked against the built library reaches the host-only entry points without a GPU."""
import os
import shutil
import subprocess

import pytest

import paper_2504_18658_amd.build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")
HEADER = os.path.join(INCLUDE, "pccl_local.h")

pytestmark = pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("gcc", "-std=c11"), ("g++", "-std=c++11"),
                                          ("g++", "-std=c++17")])
def test_header_compiles_alone_in_strict_mode(tmp_path, compiler, std):
    lang = "c" if compiler == "gcc" else "c++"
    src = tmp_path / ("only_header." + ("c" if lang == "c" else "cpp"))
    src.write_text('#include "pccl_local.h"\n#include "pccl_local.h"\nint unused_symbol_to_make_a_unit;\n')
    subprocess.check_call([compiler, std, "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-I", INCLUDE,
                           "-c", str(src), "-o", str(tmp_path / "only_header.o")])


def test_c_program_links_and_calls_host_paths(tmp_path):
    if not os.path.exists(B.LIB):
        pytest.skip("library not built")
    exe = tmp_path / "abi_c_main"
    libdir = os.path.dirname(B.LIB)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-I", INCLUDE,
                           os.path.join(ROOT, "tests", "abi_c_main.c"), "-o", str(exe),
                           "-L", libdir, "-l:libpccl_local.so", "-Wl,-rpath," + libdir, "-lm"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "abi_c_main: ok" in out.stdout
