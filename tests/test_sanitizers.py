"""CPU sanitizer legs (AddressSanitizer + UndefinedBehaviorSanitizer, host code
only): the oracle's C source driven over small layers with its edge cases, and
the library's host-side argument validation / workspace carving with the kernel
launchers stubbed out.  Both are standalone executables built here; nothing
runs on a GPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    return p.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-std=c11", *SAN,
                           "-o", exe, os.path.join(ROOT, "oracle", "moe_oracle.c"),
                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-lm"])
    assert "ok" in _run(exe)


def test_host_validation_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "api_san")
    host = [a for s in SAN for a in ("-Xarch_host", s)]
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host,
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2601_08800_amd", "csrc"),
                           os.path.join(ROOT, "paper_2601_08800_amd", "csrc", "moe_api.hip"),
                           os.path.join(ROOT, "tests", "sanitize", "api_driver.cpp"), "-o", exe],
                          stderr=subprocess.DEVNULL)
    assert "ok" in _run(exe)
