"""CPU sanitizer leg: the scalar C oracle and the host side of the C ABI (argument validation) built with the address and
undefined-behaviour sanitizers and run as plain executables.  Nothing here touches a GPU; device code is not instrumented."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_oracle_selfcheck_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "selfcheck")
    _run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", os.path.join(ROOT, "oracle", "selfcheck_w4.c"), os.path.join(ROOT, "oracle", "oracle_w4.c"),
          "-lm", "-o", exe])
    assert "all checks passed" in _run([exe], env=ENV)


def test_abi_argument_validation_under_asan_ubsan(tmp_path):
    from paper_2508_15601_amd import build as B
    objdir = os.path.join(B.PKG, "_build")
    others = [os.path.join(objdir, s.replace(".hip", ".o")) for s in B.SOURCES if s != "tm_w4_api.hip"]
    if not all(os.path.exists(o) for o in others):
        B.build()                                  # the kernels' objects are linked in as they are (uninstrumented)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", B.CSRC]
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    api = str(tmp_path / "api_san.o")
    _run([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument", *san_host, *inc, "-c", os.path.join(B.CSRC, "tm_w4_api.hip"), "-o", api])
    drv = str(tmp_path / "drv.o")
    _run([hipcc, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all",
          "-fno-gpu-sanitize", *inc, "-x", "c++", "-c", os.path.join(ROOT, "tests", "abi_args_check.cpp"), "-o", drv])
    exe = str(tmp_path / "abi_args_check")
    _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", drv, api, *others, "-o", exe])
    assert "all checks passed" in _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
