"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU side (no GPU needed): the float64 oracle on small
inputs with its edge cases, and the host side of the C ABI (argument validation, workspace arithmetic).  Both are
standalone executables (tests/sanitizer/*), so nothing is preloaded into this process."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitizer")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="2")


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, f"{exe} failed ({r.returncode}):\n{r.stdout[-2000:]}\n{r.stderr[-6000:]}"
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-6000:]
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall",
                           os.path.join(ROOT, "oracle", "criticalkv_oracle.c"), os.path.join(SAN, "oracle_driver.c"),
                           "-o", exe, "-lm"])
    assert "OK" in _run(exe)


def test_c_abi_host_side_under_sanitizers(tmp_path):
    """api.hip's host pass is compiled with the sanitizers (device code is not instrumented) and linked with the
    other kernel objects and a driver that only makes calls the validation refuses."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2502_03805_amd import build as B
    objs = sorted(glob.glob(os.path.join(B.PKG, "_build", "*.hip.o")))
    if len(objs) != len(B.sources()):
        B.build(force=True)
        objs = sorted(glob.glob(os.path.join(B.PKG, "_build", "*.hip.o")))
    others = [o for o in objs if not o.endswith("api.hip.o")]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all"]
    api_o = str(tmp_path / "api_san.o")
    subprocess.check_call([hipcc, *B.FLAGS, "-g", *san, "-c", os.path.join(B.CSRC, "api.hip"), "-o", api_o],
                          stderr=subprocess.DEVNULL)
    drv_o = str(tmp_path / "abi_driver.o")
    subprocess.check_call(["/opt/rocm/llvm/bin/clang++", "-std=c++17", "-O1", "-g",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include"),
                           "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv_o])
    exe = str(tmp_path / "abi_asan")
    subprocess.check_call(["/opt/rocm/llvm/bin/clang++", "-fsanitize=address,undefined", api_o, drv_o, *others, "-o", exe,
                           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    assert "OK" in _run(exe)
