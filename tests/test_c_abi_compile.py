"""The boundary is a C ABI: a C11 program compiled with gcc against include/tpo.h (and
include/tpo_bench.h for the measurement aid) links with libtpo.so (and libtpo_bench.so) and
gets the documented statuses from argument validation (no GPU needed)."""
import os
import shutil
import subprocess

import pytest

from paper_2604_19906_amd import tpo


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_c_program_links_and_validates(repo_root, tmp_path):
    tpo.lib()                                            # raises if the library is not built
    tpo.bench_lib()
    libdir = os.path.dirname(tpo.LIB_PATH)
    exe = str(tmp_path / "abi_check")
    src = os.path.join(repo_root, "tests", "c_abi", "abi_check.c")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(repo_root, "include"), src, "-o", exe,
                    "-L", libdir, "-ltpo", "-ltpo_bench", f"-Wl,-rpath,{libdir}"], check=True)
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = libdir + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
