"""Host-side AddressSanitizer + UndefinedBehaviorSanitizer builds (CPU only, no GPU code is
instrumented): the C oracle with a driver that calls every one of its entry points on exactly sized
buffers, and the library's argument-validation code (csrc/fmt_api.hip, host pass only) with a driver
that makes every entry point refuse bad arguments.  Any sanitizer finding aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=99", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "fmt_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"]
    p = run(cmd)
    assert p.returncode == 0, p.stdout
    p = run([exe], env=dict(ENV, OMP_NUM_THREADS="2"), timeout=300)
    assert p.returncode == 0 and "oracle sanitizer run ok" in p.stdout, p.stdout[-3000:]


def test_library_argument_validation_under_asan_and_ubsan(tmp_path):
    from paper_2103_15940_amd import build as b
    hipcc = b.hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    objs = [os.path.join(b.CSRC, s.replace(".hip", ".o")) for s in b.SOURCES if s != "fmt_api.hip"]
    if not all(os.path.exists(o) for o in objs):
        pytest.skip("the library has not been built here (its object files are linked in)")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    api_o = str(tmp_path / "fmt_api_san.o")
    p = run([hipcc, *b.FLAGS, "-g", *san, "-I", os.path.join(ROOT, "include"), "-I", b.CSRC,
             "-c", os.path.join(b.CSRC, "fmt_api.hip"), "-o", api_o])
    assert p.returncode == 0, p.stdout[-3000:]
    lib = str(tmp_path / "libfmt_san.so")
    p = run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
             "-shared-libsan", "-o", lib, api_o, *objs])
    assert p.returncode == 0, p.stdout[-3000:]
    exe = str(tmp_path / "abi_san")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    p = run([clang, "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libsan",
             "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "abi_driver.c"), "-o", exe,
             "-L", str(tmp_path), "-lfmt_san", "-Wl,-rpath," + str(tmp_path)])
    assert p.returncode == 0, p.stdout[-3000:]
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    env = dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"] + ":verify_asan_link_order=0:detect_leaks=0")
    env["LD_LIBRARY_PATH"] = os.path.dirname(rt) + ":" + env.get("LD_LIBRARY_PATH", "")
    p = run([exe], env=env, timeout=300)
    assert p.returncode == 0 and "abi sanitizer run ok" in p.stdout, p.stdout[-3000:]
