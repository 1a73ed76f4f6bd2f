"""Host sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer), CPU only: the C oracles under gcc, and the
C-ABI layer of the library (argument validation, size arithmetic, workspace carving: everything that runs before a
kernel is enqueued) under hipcc with the sanitizers on the host side only.  Each is a small driver program under
tests/sanitize/ that aborts on the first finding."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)          # the AddressSanitizer runtime insists on being the first library


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


def test_oracles_under_host_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "conv2d_direct.c"),
          os.path.join(ROOT, "oracle", "conv2d_general.c"), "-lm", "-o", exe])
    out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=0"))      # libgomp keeps its thread pool
    assert "oracle sanitizer run ok" in out


def test_abi_layer_under_host_sanitizers(tmp_path):
    from paper_2412_05781_amd import build as bld
    bld.build_libwino(incremental=True)              # the kernels' objects (not instrumented; only the ABI layer is)
    api_obj = str(tmp_path / "wino_api_san.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    _run([bld.HIPCC] + bld.CFLAGS + ["-g", "-fno-omit-frame-pointer"] + san + ["-c", os.path.join(bld.CSRC, "wino_api.hip"), "-o", api_obj])
    drv_obj = str(tmp_path / "abi_driver.o")
    _run([bld.HIPCC, "-std=c++17", "-O1", "-g", "-x", "c++", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-I" + os.path.join(ROOT, "include"), "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv_obj])
    others = [os.path.join(bld.OBJ, os.path.basename(s)[:-4] + ".o") for s in bld.sources() if not s.endswith("wino_api.hip")]
    exe = str(tmp_path / "abi_driver")
    _run([bld.HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-Wno-unused-command-line-argument",
          drv_obj, api_obj] + others + ["-o", exe])
    out = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))       # the HIP runtime's start-up allocations are not ours
    assert "abi sanitizer run ok" in out
