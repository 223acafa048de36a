"""AddressSanitizer + UndefinedBehaviorSanitizer builds (host compiler, CPU only) of the two bodies of host code
the parity claims lean on: the oracle, walked by oracle/sanitize_check.cpp, and the library's host-only
translation unit (validation, sizes, Table 1, Theorem 2's condition, code construction of the entropy coder),
walked by tests/host_sanitize_check.cpp.  A report from either sanitizer ends the program with a non-zero status."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
       "-fno-omit-frame-pointer", "-ffp-contract=off", "-Wall"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the program's library list


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    odir = os.path.join(ROOT, "oracle")
    srcs = [os.path.join(odir, s) for s in ("sanitize_check.cpp", "lpco_philox.cpp", "lpco_quant.cpp", "lpco_glm.cpp",
                                            "lpco_mlp.cpp", "lpco_svrg.cpp")]
    exe = str(tmp_path / "oracle_san")
    subprocess.run(SAN + ["-fopenmp", "-I", odir, "-o", exe] + srcs, check=True)
    assert "oracle sanitizer walk: ok" in _run(exe)


def test_library_host_code_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_1901_08924_amd", "csrc")
    exe = str(tmp_path / "host_san")
    # the HIP runtime's headers are needed for the types of the internal header only: nothing of HIP is linked
    subprocess.run(SAN + ["-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
                          "-I", csrc, "-o", exe, os.path.join(csrc, "lpc_host.cpp"),
                          os.path.join(ROOT, "tests", "host_sanitize_check.cpp")], check=True)
    assert "host sanitizer walk: ok" in _run(exe)
