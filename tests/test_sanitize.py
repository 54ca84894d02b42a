"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code (CPU only, no GPU work):
  * the oracle, driven by oracle/sanitize_driver.cpp through every exported function at the shapes of the pin
    suite's heaviest cases;
  * the library's host-only paths (append planner, argument checks that return before any GPU call), from the
    host pass of csrc/specache.hip and csrc/measure.hip, driven by tests/host/host_sanitize_driver.cpp.
A sanitizer report aborts the driver, which fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    assert r.returncode == 0, f"{' '.join(cmd[:3])} ... failed ({r.returncode}):\n{r.stdout[-2000:]}\n{err[-4000:]}"
    return r.stdout


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    _run(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", "-o", exe,
          os.path.join(ROOT, "oracle", "specache_oracle.cpp"), os.path.join(ROOT, "oracle", "sanitize_driver.cpp")])
    assert "sanitize_driver ok" in _run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc for the host pass of the .hip sources")
def test_library_host_paths_under_address_and_undefined_sanitizers(tmp_path):
    from paper_2503_16163_amd import build as hip_build
    if not hip_build.is_built():
        hip_build.build()     # the kernels' objects are linked as they are; only the host code is instrumented
    csrc = os.path.join(ROOT, "paper_2503_16163_amd", "csrc")
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Xclang", "-target-feature",
             "-Xclang", "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    objs = []
    for src, lang in ((os.path.join(csrc, "specache.hip"), []), (os.path.join(csrc, "measure.hip"), []),
                      (os.path.join(ROOT, "tests", "host", "host_sanitize_driver.cpp"), ["-x", "hip"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        _run(["hipcc", *flags, *lang, "-c", src, "-o", obj])
        objs.append(obj)
    others = [os.path.join(hip_build.OBJ, s.replace(".hip", ".o")) for s in hip_build.SOURCES
              if s not in ("specache.hip", "measure.hip")]
    exe = str(tmp_path / "host_sanitize")
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe,
          *objs, *others])
    assert "host_sanitize_driver ok" in _run([exe], env=ENV)
