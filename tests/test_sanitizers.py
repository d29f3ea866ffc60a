"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU needed): the
oracle with a driver that walks all its entry points on exact-size buffers, and the library's host
side (planning, argument validation: everything that returns before the first HIP call) with a
driver of its own.  Device code is compiled as usual and never runs here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
# the sanitizer runtime need not be first among the preloaded libraries of the test process
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    run(["gcc", "-O1", "-g", "-fopenmp", *SAN, os.path.join(ROOT, "oracle", "tlin_oracle.c"),
         os.path.join(NATIVE, "oracle_driver.c"), "-lm", "-o", exe])
    r = run([exe], env=ENV, timeout=300)
    assert "oracle driver ok" in r.stdout and "runtime error" not in r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_library_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    obj, drv, exe = (str(tmp_path / n) for n in ("tlinattn_asan.o", "driver.o", "host_api_asan"))
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2508_20407_amd", "csrc")]
    # sanitizers on the host pass only: each -fsanitize= directly behind its own -Xarch_host
    run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
         "-Xarch_host", "-fno-sanitize-recover=undefined", *inc,
         "-c", os.path.join(ROOT, "paper_2508_20407_amd", "csrc", "tlinattn.hip"), "-o", obj], cwd=str(tmp_path))
    clang = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    run([clang, "-O1", "-g", *SAN, *inc, "-c", os.path.join(NATIVE, "host_api_driver.c"), "-o", drv])
    # link only (no device compile on this line): the sanitizer runtimes for the host objects
    run(["hipcc", "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address,undefined", obj, drv, "-o", exe],
        cwd=str(tmp_path))
    r = run([exe], env=dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")), timeout=300)
    assert "host api driver ok" in r.stdout and "runtime error" not in r.stderr
