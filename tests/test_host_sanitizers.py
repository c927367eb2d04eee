"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, nothing is launched).

  * the C oracle, built whole with the sanitizers and driven through every routine and argument form by
    tests/sanitize/oracle_driver.c; its printed results must equal the ordinary build's;
  * the C ABI's argument layer (csrc/loma_api.hip and the split planning of csrc/loma_decode.hip, host side
    only: the device code is compiled as always) driven by tests/sanitize/abi_driver.cpp through rejected calls
    and host-only queries; the kernel-heavy translation units are linked from the library's ordinary objects.
Executables carry the sanitizer runtimes statically, so they run next to whatever the environment preloads.
"""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    assert res.returncode == 0, f"{' '.join(cmd[:3])} ... failed ({res.returncode}):\n{res.stdout[-2000:]}\n{err[-4000:]}"
    return res.stdout, err


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_sanitizers(tmp_path, c_oracle):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-static-libasan", "-fopenmp", "-std=c11", "-Wall", "-Wextra", os.path.join(SAN, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "loma_oracle.c"), "-o", exe, "-lm"])
    out, err = run([exe], env=ENV)
    assert "oracle driver ok" in out and "runtime error" not in err and "AddressSanitizer" not in err
    # the same driver against the ordinary build of the oracle: identical numbers
    plain = str(tmp_path / "oracle_plain")
    run(["gcc", "-O2", "-fopenmp", "-std=c11", os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "loma_oracle.c"),
         "-o", plain, "-lm"])
    out2, _ = run([plain])
    a = [ln.split() for ln in out.splitlines() if " " in ln and not ln.startswith("oracle")]
    b = [ln.split() for ln in out2.splitlines() if " " in ln and not ln.startswith("oracle")]
    assert len(a) == len(b) == 2 * 10
    for la, lb in zip(a, b):
        assert la[0] == lb[0]
        np.testing.assert_allclose(np.array(la[1:], dtype=np.float64), np.array(lb[1:], dtype=np.float64), rtol=1e-13, atol=1e-15)


def test_abi_argument_layer_under_sanitizers(tmp_path):
    from paper_2401_09486_amd import build as hb
    if not os.path.exists(hb.HIPCC):
        pytest.skip("hipcc not available")
    others = [os.path.join(hb.OBJDIR, os.path.splitext(s)[0] + ".o") for s in hb.SOURCES if s not in ("loma_api.hip", "loma_decode.hip")]
    if not all(os.path.exists(o) for o in others):
        pytest.skip("library objects not built (python -m paper_2401_09486_amd.build)")
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-fPIC", "-std=c++17", "-fno-omit-frame-pointer",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san_host]
    objs = []
    for src in ("loma_api.hip", "loma_decode.hip"):
        obj = str(tmp_path / (src + ".o"))
        run([hb.HIPCC, *flags, "-c", os.path.join(hb.CSRC, src), "-o", obj])
        objs.append(obj)
    drv = str(tmp_path / "drv.o")
    clangxx = os.path.join(os.path.dirname(os.path.realpath(hb.HIPCC)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    run([clangxx, "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-c",
         os.path.join(SAN, "abi_driver.cpp"), "-o", drv])
    exe = str(tmp_path / "abi_san")
    run([hb.HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", drv, *objs, *others, "-o", exe])
    out, err = run([exe], env=ENV)
    assert "abi driver ok" in out and "runtime error" not in err and "AddressSanitizer" not in err
