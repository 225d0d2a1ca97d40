"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no device is touched): the C oracle in both
precisions driven over every entry point, and the host side of the C ABI (a copy of the library whose host code is
instrumented) walked through every call it must answer before it reaches a device.  The drivers are standalone
programs under tests/sanitize/: nothing is preloaded into the Python process."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2509_18362_amd import build as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{err}"
    return res.stdout


@pytest.mark.parametrize("precision_flag", [[], ["-DORC_F64"]], ids=["f32", "f64"])
def test_oracle_under_sanitizers(precision_flag):
    with tempfile.TemporaryDirectory(prefix="mtp_san_") as tmp:
        exe = os.path.join(tmp, "oracle_san")
        run(["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", *precision_flag, os.path.join(SAN, "oracle_driver.c"), "-lm", "-o", exe])
        assert "ok" in run([exe], env=ENV)


def test_host_abi_under_sanitizers():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    with tempfile.TemporaryDirectory(prefix="mtp_san_") as tmp:
        objs = [os.path.join(tmp, os.path.splitext(src)[0] + ".o") for src in b.SOURCES]
        # -O1: the device code is not run here, only compiled along
        flags = [f for f in b.HIPCC_FLAGS if f != "-O3"] + ["-O1"]
        cmds = [[hipcc, *flags, *san, "-c", os.path.join(b.CSRC, src), "-o", obj] for src, obj in zip(b.SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=len(cmds)) as pool:
            list(pool.map(run, cmds))
        lib = os.path.join(tmp, "libmtp_draft_san.so")
        link = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-shared-libsan"]
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *link, *objs, "-o", lib])
        exe = os.path.join(tmp, "abi_san")
        clangxx = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang++")
        rt = os.path.dirname(run([clangxx, "-print-file-name=libclang_rt.asan-x86_64.so"]).strip())
        # (the driver is plain C++; hipcc compiles it as a HIP source with no kernels, which keeps one toolchain and one
        # sanitizer runtime for the program and the library)
        obj = os.path.join(tmp, "abi_driver.o")
        run([hipcc, "--offload-arch=gfx950", "-std=c++17", "-O1", *san, "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", obj])
        run([hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", *link, obj, lib, f"-Wl,-rpath,{tmp}", f"-Wl,-rpath,{rt}",
             "-o", exe])
        assert "ok" in run([exe], env=ENV)
