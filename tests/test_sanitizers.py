"""Sanitizer leg (CPU only): the oracle and the library's host code under AddressSanitizer and
UndefinedBehaviorSanitizer.

Two builds with clang -fsanitize=address,undefined:
  * oracle/qtip_oracle.c (plain C, without OpenMP);
  * the host side of the library: qtip_api.hip (argument checks and dispatch, compiled as C++)
    and qtip_quantize.cpp (the host Viterbi quantizer), linked with tests/sanitize/stub_launchers.cpp
    in place of the kernel launchers, so no GPU and no HIP runtime is involved.
A child pytest process then runs the oracle pins, the host-quantizer tests and the argument-error
cases against those two builds (QTIP_ORACLE_LIBRARY, QTIP_LIBRARY) with the sanitizer runtime
preloaded; any report aborts the child (-fno-sanitize-recover).  Leak checking is off: the
interpreter itself never frees everything.

The two slowest cases are left out by default; QTIP_SANITIZE=full runs them too (about 80 s).
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2406_11235_amd", "csrc")
CLANG = os.environ.get("QTIP_CLANG", "/opt/rocm/lib/llvm/bin/clang")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan", "-g", "-O1", "-fPIC"]


def asan_runtime():
    out = subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = out.stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    if not os.path.exists(CLANG) or asan_runtime() is None:
        pytest.skip("no clang with a shared AddressSanitizer runtime")
    out = tmp_path_factory.mktemp("san")
    # (the two macros are the ones a plain C++ compile of the HIP headers leaves undefined)
    cxx = [CLANG + "++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-D__align__(n)=__attribute__((aligned(n)))",
           "-DHIP_SYMBOL(x)=x", "-I/opt/rocm/include", "-I" + CSRC] + SAN
    objs = []
    for src, extra in (("qtip_api.hip", ["-x", "c++"]), ("qtip_quantize.cpp", ["-pthread"]),
                       (os.path.join(ROOT, "tests", "sanitize", "stub_launchers.cpp"), [])):
        obj = str(out / (os.path.basename(src).split(".")[0] + ".o"))
        subprocess.run(cxx + extra + ["-c", os.path.join(CSRC, src), "-o", obj], check=True)
        objs.append(obj)
    host = str(out / "libqtip_host_san.so")
    subprocess.run([CLANG + "++", "-shared", "-pthread"] + SAN + objs + ["-o", host], check=True)
    orc = str(out / "libqtip_oracle_san.so")
    subprocess.run([CLANG, "-std=c11", "-ffp-contract=off", "-shared"] + SAN +
                   [os.path.join(ROOT, "oracle", "qtip_oracle.c"), "-o", orc, "-lm"], check=True)
    return host, orc


def test_oracle_and_host_code_are_clean_under_asan_and_ubsan(sanitized):
    host, orc = sanitized
    env = dict(os.environ)
    preload = [asan_runtime()] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env.update(LD_PRELOAD=":".join(preload), ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", QTIP_ORACLE_LIBRARY=orc, QTIP_LIBRARY=host)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           "tests/test_abi.py::test_argument_errors_need_no_gpu", "tests/test_host_quantizer.py",
           "tests/test_oracle_pins.py"]
    if os.environ.get("QTIP_SANITIZE") != "full":
        cmd += ["--deselect", "tests/test_host_quantizer.py::test_quantizer_matches_oracle_algorithm4[2-4-2]",
                "--deselect", "tests/test_oracle_pins.py::test_paper_mse_tables_loose"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
