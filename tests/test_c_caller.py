"""The boundary is a C ABI: a plain C99 program (tests/c_caller.c) includes include/mpq.h, links
against libmpq.so and calls it -- host functions and argument checks only, so it runs without a GPU."""
import os
import shutil
import subprocess

import pytest

from paper_2302_01382_amd import build

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_a_c_program_links_and_calls_the_library(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    if build.is_stale():
        build.build_lib()
    libdir = os.path.dirname(build.LIB)
    exe = str(tmp_path / "c_caller")
    rocm_lib = "/opt/rocm/lib"
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "c_caller.c"), "-o", exe, "-L", libdir, "-l:" + os.path.basename(build.LIB),
           "-Wl,-rpath," + libdir, "-Wl,-rpath-link," + rocm_lib, "-Wl,-rpath," + rocm_lib]
    if build.SANITIZE_HOST:   # the instrumented library needs the sanitizer runtimes in the program too
        # (the library was instrumented by clang, the runtimes here are gcc's: symbols that only clang's
        # runtime has stay unresolved, as they do when Python loads the library)
        cmd += ["-fsanitize=address,undefined", "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0 and "c caller ok" in r.stdout, r.stdout
