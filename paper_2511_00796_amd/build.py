"""Builds libhexdecode.so from csrc/ with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libhexdecode.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "kv_cache.hip", "attention.hip", "attention_chunk.hip", "attention_fp8.hip", "gemm.hip", "gemm_wide.hip", "elementwise.hip", "sampling.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off: products and sums round separately unless fmaf is written out;
# packed fp32 instructions are switched off for the device pass.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


# host-side sanitizers (address + undefined behaviour) for the CPU check of the library's host logic; device code is
# compiled as usual (every -fsanitize= directly behind -Xarch_host)
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def compiler_id() -> str:
    """The device compiler's identity: the 'clang version' line of `hipcc --version` (vendor, version, revision)."""
    r = subprocess.run([HIPCC, "--version"], capture_output=True, text=True)
    for line in r.stdout.splitlines():
        if "clang version" in line:
            return line.strip()
    return "unknown: " + (r.stdout + r.stderr).strip()[:200]


def _compile(src: str, sanitize: bool = False) -> str:
    obj = os.path.join(OBJ_DIR + ("_hostsan" if sanitize else ""), src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *(SAN_FLAGS if sanitize else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False, sanitize: bool = False) -> str:
    """sanitize: a second library, libhexdecode_hostsan.so, whose HOST code carries AddressSanitizer and
    UndefinedBehaviorSanitizer checks (loaded only by the sanitizer test's driver program, never by the binding)."""
    out = OUT.replace(".so", "_hostsan.so") if sanitize else OUT
    os.makedirs(OBJ_DIR + ("_hostsan" if sanitize else ""), exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, sanitize), SOURCES))
    tmp = out + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *(["-fsanitize=address,undefined", "-shared-libsan"] if sanitize else []),
                        *objs, "-o", tmp], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, out)
    with open(out + ".compiler.txt", "w") as f:      # which compiler produced the library that is loaded
        f.write(compiler_id() + "\n")
    if verbose:
        print("built", out, "with", compiler_id())
    return out


if __name__ == "__main__":
    build(verbose=True, sanitize="--sanitize" in sys.argv[1:])
