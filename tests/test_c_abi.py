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
    # the ctypes mirrors of the structs have the sizes the C compiler gives them
    import ctypes as C
    import re
    from paper_2402_02447_amd import binding, lbs
    sizes = dict(re.findall(r"(\w+) (\d+)", r.stdout.split("sizeof", 1)[1].splitlines()[0]))
    assert int(sizes["bca_segment"]) == C.sizeof(binding._Segment) and int(sizes["bca_tuning"]) == C.sizeof(binding._Tuning)
    assert int(sizes["bca_adam"]) == C.sizeof(binding._Adam) and int(sizes["lbs_run"]) == C.sizeof(lbs._Run)


def _torch_lib_env():
    env = dict(os.environ)
    try:
        import torch
        env["LD_LIBRARY_PATH"] = os.path.join(os.path.dirname(torch.__file__), "lib") + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    except ImportError:
        env["LD_LIBRARY_PATH"] = "/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    return env


def test_host_side_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    # The library's host code (plan construction, validation, table building) rebuilt with ASan + UBSan on the host
    # pass only (device code is compiled as usual), driven by the same C program; leaks count as failures.
    from paper_2402_02447_amd import build as lib_build
    san = str(tmp_path / "libbca_san.so")
    extra = ["-O1", "-g"]
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        extra += ["-Xarch_host", f]
    lib_build.build(extra=extra, out=san)
    exe = str(tmp_path / "host_check_san")
    clang = "/opt/rocm/lib/llvm/bin/clang"
    subprocess.run([clang, "-std=c99", "-g", "-fsanitize=address,undefined", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi", "host_check.c"), "-o", exe, "-L", str(tmp_path), "-l:libbca_san.so",
                    f"-Wl,-rpath,{tmp_path}", "-Wl,--allow-shlib-undefined"], check=True)
    env = _torch_lib_env()
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "c abi ok" in r.stdout, r.stdout + r.stderr[-3000:]


def test_oracles_are_clean_under_the_undefined_behaviour_sanitizer(tmp_path):
    # Both oracles rebuilt with UBSan (traps on the first report) and put through a sample of their pin tests.
    import sys
    from oracle import build as obuild
    env = dict(os.environ)
    for src, name, var in ((obuild.SRC, "libbca_oracle_ub.so", "BCA_ORACLE_LIB"), (obuild.LBS_SRC, "liblbs_oracle_ub.so", "LBS_ORACLE_LIB")):
        out = str(tmp_path / name)
        subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fsanitize=undefined",
                        "-fno-sanitize-recover=all", "-o", out, src], check=True)
        env[var] = out
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_norm_clip.py",
                        "tests/test_oracle_lamb.py", "tests/test_oracle_lbs.py", "tests/test_oracle_bf16.py", "tests/test_golden.py"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
