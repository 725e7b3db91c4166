"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU code is
instrumented): the C oracle, and the library's host side (dictionary, encoder, validation,
argument checks, launch planning).  Each leg builds a sanitized copy and re-runs the existing
host tests against it in a child process that preloads the sanitizer's runtime; any report
makes the child exit non-zero.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2310_16795_amd", "csrc")


def _run_child(files, env_extra, preload):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = " ".join(x for x in (env.get("LD_PRELOAD"), preload) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=23"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=23"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "passed" in r.stdout


def test_oracle_under_asan_and_ubsan():
    rt = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("gcc's libasan is not installed")
    env = {"ORACLE_SANITIZE": "1"}
    subprocess.check_call([sys.executable, "-c", "import oracle; oracle.build()"], cwd=ROOT, env={**os.environ, **env})
    _run_child(["tests/test_oracle_codec.py", "tests/test_oracle_dictionary.py", "tests/test_oracle_matvec.py"], env, rt)


def test_library_host_side_under_asan_and_ubsan():
    from paper_2310_16795_amd import build as B

    cands = []
    for base, _, files in os.walk("/opt/rocm/lib/llvm/lib/clang"):
        cands += [os.path.join(base, f) for f in files if f == "libclang_rt.asan-x86_64.so"]
    if not cands:
        pytest.skip("clang's shared ASan runtime is not installed")
    B.build_library(incremental=True)  # the device objects the sanitized host objects are linked with
    san = os.path.join(B.OBJ, "san")
    os.makedirs(san, exist_ok=True)
    host_flags = ["-O1", "-g", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    subprocess.check_call(["hipcc", *host_flags, "-fsanitize=address", "-fsanitize=undefined",
                           "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize",
                           "-c", os.path.join(CSRC, "qmoe_host.cpp"), "-o", os.path.join(san, "qmoe_host.o")])
    subprocess.check_call(["hipcc", *host_flags, "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=undefined",
                           "-c", os.path.join(CSRC, "qmoe_api.hip"), "-o", os.path.join(san, "qmoe_api.o")],
                          stderr=subprocess.DEVNULL)
    others = [os.path.join(B.OBJ, os.path.splitext(u)[0] + ".o") for u in B.UNITS
              if u not in ("qmoe_host.cpp", "qmoe_api.hip")]
    lib = os.path.join(san, "libqmoe_san.so")
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address",
                           "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize", "-o", lib,
                           os.path.join(san, "qmoe_host.o"), os.path.join(san, "qmoe_api.o"), *others])
    _run_child(["tests/test_lib_host.py"], {"QMOE_LIBRARY": lib}, cands[0])
