"""The two headers are plain C and the library can be driven from a C program: tests/c_abi/host_check.c is
compiled with gcc as C99, linked against libbca.so and run (host-only plans, no GPU)."""
import os
import subprocess

import paper_2402_02447_amd as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c99_program_builds_against_the_headers_and_runs(tmp_path):
    lib = B.library_path()
    assert os.path.exists(lib), "build libbca.so first"
    exe = str(tmp_path / "host_check")
    src = os.path.join(ROOT, "tests", "c_abi", "host_check.c")
    libdir = os.path.dirname(lib)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), src,
                    "-o", exe, "-L", libdir, "-l:libbca.so", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,--allow-shlib-undefined"],
                   check=True)
    env = dict(os.environ)
    # the library's HIP runtime: the copy torch ships when present (as the Python binding uses), else ROCm's
    try:
        import torch
        env["LD_LIBRARY_PATH"] = os.path.join(os.path.dirname(torch.__file__), "lib") + ":" + env.get("LD_LIBRARY_PATH", "")
    except ImportError:
        pass
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "c abi ok" in r.stdout, r.stdout + r.stderr
