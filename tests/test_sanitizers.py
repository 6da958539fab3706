"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the code that executes on the host, on the CPU:

  * the oracle (oracle/decode_oracle.c), driven through every entry point by tests/sanitize/oracle_driver.c;
  * the library's host logic -- size queries, buffer maps, argument validation, the launch planner -- built from
    the same csrc/*.hip with sanitizers on the host side only (build.py --sanitize) and driven by
    tests/sanitize/host_abi_driver.cpp.  No kernel is launched, no GPU is needed.

A sanitizer report aborts the driver (no recovery), so a non-zero exit status or any report text fails the test."""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def run_clean(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    text = r.stdout + r.stderr
    assert r.returncode == 0, text[-3000:]
    assert "Sanitizer" not in text and "runtime error" not in text, text[-3000:]
    return text


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_driver")
        run_clean(["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", *SAN, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                   os.path.join(ROOT, "oracle", "decode_oracle.c"), "-o", exe, "-lm"])
        out = run_clean([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="4"))
        assert "oracle sanitizer driver: OK" in out


def test_library_host_logic_under_address_and_undefined_behaviour_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2511_00796_amd import build as hip_build
    lib = hip_build.OUT.replace(".so", "_hostsan.so")
    srcs = [os.path.join(hip_build.CSRC, f) for f in os.listdir(hip_build.CSRC)] + [os.path.join(ROOT, "include", "hexdecode.h")]
    if not os.path.exists(lib) or os.path.getmtime(lib) < max(os.path.getmtime(f) for f in srcs):
        hip_build.build(sanitize=True)
    clang = os.path.join(os.path.dirname(os.path.realpath(hip_build.HIPCC)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang++"
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_abi_driver")
        run_clean([clang, "-std=c++17", *SAN, "-shared-libsan", os.path.join(ROOT, "tests", "sanitize", "host_abi_driver.cpp"), lib,
                   "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath," + os.path.dirname(rt), "-o", exe])
        # leak detection off: the HIP runtime, which the library links, keeps its own allocations until exit
        out = run_clean([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
        assert "host ABI sanitizer driver: OK" in out
