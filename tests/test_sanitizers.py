"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code, on the CPU:

  * the oracle (oracle/nqkv_oracle.cpp compiled into tests/sanitize/oracle_driver.cpp), every entry
    point on small inputs;
  * the host layer of the library (csrc/nqkv_host.cpp: validation, quantile table, split and page
    planning, table scaling, the quantizer's cell table) built as plain C++ against stub kernel
    launchers (tests/sanitize/launch_stubs.cpp) and driven through the C ABI by
    tests/sanitize/host_driver.cpp -- every geometry, every entry point, every refusal.

Sanitizers cannot run on this GPU pool's device code; these cover what runs on the host."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-ffp-contract=off"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _have_sanitizers(tmp_path) -> bool:
    if shutil.which("g++") is None:
        return False
    src = tmp_path / "probe.cpp"
    src.write_text("int main() { return 0; }\n")
    r = subprocess.run(["g++", *SAN, str(src), "-o", str(tmp_path / "probe")], capture_output=True)
    return r.returncode == 0


def test_oracle_under_asan_ubsan(tmp_path):
    if not _have_sanitizers(tmp_path):
        pytest.skip("g++ with the sanitizer runtimes is not available")
    exe = tmp_path / "oracle_driver"
    subprocess.run(["g++", *SAN, "-pthread", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.cpp"), "-o", str(exe)],
                   check=True, capture_output=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "oracle sanitizer run: ok" in r.stdout


def test_host_layer_under_asan_ubsan(tmp_path):
    if not _have_sanitizers(tmp_path):
        pytest.skip("g++ with the sanitizer runtimes is not available")
    if not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"):
        pytest.skip("HIP headers are not installed")
    exe = tmp_path / "host_driver"
    srcs = [os.path.join(ROOT, "paper_2505_16210_amd", "csrc", "nqkv_host.cpp"),
            os.path.join(ROOT, "tests", "sanitize", "launch_stubs.cpp"),
            os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp")]
    cmd = ["g++", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-w", "-x", "c++", *srcs, "-o", str(exe),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host-layer sanitizer run: ok" in r.stdout
