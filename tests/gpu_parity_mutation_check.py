"""Sensitivity of the GPU parity tests, by mutation of the ORACLE (needs a GPU; the kernels are never changed): plants
one mistake at a time (the list of oracle_mutation_check.py) in a scratch copy of oracle/decode_oracle.c and runs the
GPU parity tests that cover the mutated function against it.  They must fail: a kernel with the same mistake would
disagree with the true oracle in the same way.  Not collected by pytest; run by hand from the repository root:

    python tests/gpu_parity_mutation_check.py

Two mutants are expected to survive: the GPU tests check the query's bf16 rounding and the arg-max tie rule against
the definition directly, not through the oracle functions these two mutants change.
"""
import os, shutil, subprocess, sys, tempfile
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "tests"))
import oracle_mutation_check as omc
DST = os.path.join(tempfile.gettempdir(), "gpu_parity_mutation_check")
SKIP = ("philox", "uniform", "sample", "top-p", "e4m3", "full causal", "argmax")   # covered by their own GPU tests below
def run():
    shutil.rmtree(DST, ignore_errors=True); os.makedirs(DST)
    ignore = shutil.ignore_patterns("liboracle*.so", "__pycache__", "_build", "*.o")
    for d in ("oracle", "tests", "paper_2511_00796_amd", "include"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(DST, d), ignore=ignore)
    src = open(DST + "/oracle/decode_oracle.c").read()
    res = []
    groups = [(m, ["tests/test_gpu_stages.py", "tests/test_gpu_decode.py"], "not full_size and not far_longer and not graph and not mid_size and not degenerate")
              for m in omc.MUT if not any(k in m[0] for k in SKIP)]
    groups += [(m, ["tests/test_gpu_sampling.py", "tests/test_gpu_top_p.py"], "not full_size and not 7b") for m in omc.MUT if any(k in m[0] for k in ("philox", "uniform", "sample", "top-p"))]
    groups += [(m, ["tests/test_gpu_fp8.py"], "not full_size and not 7b and not mid_size") for m in omc.MUT if "e4m3" in m[0]]
    groups += [(m, ["tests/test_gpu_stages.py"], "argmax or lm_head") for m in omc.MUT if "argmax" in m[0]]
    groups += [(m, ["tests/test_gpu_prefill.py", "tests/test_gpu_decode.py"], "long_prompt or chunked") for m in omc.MUT if "full causal" in m[0]]
    for (name, old, new), files, kexpr in groups:
        open(DST + "/oracle/decode_oracle.c", "w").write(src.replace(old, new, 1))
        for f in ("liboracle.so", "liboracle_desc.so"):
            try: os.remove(DST + "/oracle/" + f)
            except OSError: pass
        r = subprocess.run([sys.executable, "-m", "pytest", *files, "-x", "-q", "-m", "gpu", "-k", kexpr, "-p", "no:cacheprovider",
                            "--timeout", "120", "--timeout-method", "thread"], cwd=DST, capture_output=True, text=True, timeout=600)
        lines = [l for l in r.stdout.splitlines() if "FAILED" in l or " passed" in l or " failed" in l]
        verdict = "caught" if r.returncode == 1 else ("NOT CAUGHT" if r.returncode == 0 else "rc=%d" % r.returncode)
        first = next((l for l in lines if "FAILED" in l), lines[-1] if lines else r.stdout[-200:])
        res.append((name, verdict, first[:120])); print(res[-1], flush=True)
        if r.returncode not in (0, 1):
            print(r.stdout[-1500:], r.stderr[-500:], flush=True)
            break
    print("caught %d of %d" % (sum(1 for r in res if r[1] == "caught"), len(res)), flush=True)


if __name__ == "__main__":
    run()
