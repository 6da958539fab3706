"""The CPU pins of the oracle, checked by mutation: ONE mistake at a time is planted in a scratch copy of
oracle/decode_oracle.c (a dropped term, a wrong sign or index, a transposed operand, a rounding mode, a generator
constant, a tie rule ...), the copy is rebuilt and the oracle's pins (tests/test_oracle_*.py) are run against it in a
child process: every planted mistake must make at least one pin fail.  CPU only; the repository is not modified.

    python tests/test_oracle_mutations.py [substring of a mutation's name]     # by hand, verbose
"""
import os, shutil, subprocess, sys, tempfile
from concurrent.futures import ThreadPoolExecutor
SRC = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MUT = [
 ("rmsnorm: sum instead of mean", "float r = 1.0f / sqrtf(ss / (float)n + eps);", "float r = 1.0f / sqrtf(ss + eps);"),
 ("rmsnorm: gain dropped", "y[i] = x[i] * r * orc_bf16_to_f32(g[i]);", "y[i] = x[i] * r;"),
 ("linear: bias dropped", "for (int n = 0; n < N; ++n) y[n] += orc_bf16_to_f32(bias[n]);", "for (int n = 0; n < N; ++n) y[n] += 0.0f;"),
 ("linear: transposed weight index", "const uint16_t *w = W + (size_t)k * N;\n        for (int n = 0; n < N; ++n) y[n] += xk * orc_bf16_to_f32(w[n]);", "for (int n = 0; n < N; ++n) y[n] += xk * orc_bf16_to_f32(W[((size_t)n * K + k) % ((size_t)K * N)]);"),
 ("rope: sign of the first output", "v[i] = a * c - b * s;", "v[i] = a * c + b * s;"),
 ("rope: sign of the second output", "v[i + half] = b * c + a * s;", "v[i + half] = b * c - a * s;"),
 ("rope: exponent -i/d", "pow((double)theta, -2.0 * (double)i / (double)d)", "pow((double)theta, -1.0 * (double)i / (double)d)"),
 ("rope: adjacent pairs", "float a = v[i], b = v[i + half];\n        v[i] = a * c - b * s;\n        v[i + half] = b * c + a * s;", "float a = v[2 * i], b = v[2 * i + 1];\n        v[2 * i] = a * c - b * s;\n        v[2 * i + 1] = b * c + a * s;"),
 ("attention: scale dropped", "s[t] = dot * scale;", "s[t] = dot;"),
 ("attention: query head -> KV head by modulo", "int kvh = h / G;\n        for (int t = 0; t < T; ++t) {", "int kvh = h % c->n_kv_heads;\n        for (int t = 0; t < T; ++t) {"),
 ("attention: new token not attended", "orc_attention(c, q, kpool, vpool, table, pos + 1, o);", "orc_attention(c, q, kpool, vpool, table, pos > 0 ? pos : 1, o);"),
 ("softmax: not normalised", "for (int i = 0; i < n; ++i) p[i] = p[i] / sum;", "(void)sum;"),
 ("silu: sigmoid only", "float orc_silu(float x) { return x / (1.0f + expf(-x)); }", "float orc_silu(float x) { return 1.0f / (1.0f + expf(-x)); }"),
 ("swiglu: gate and up swapped", "gt[i] = round_act(c, orc_silu(gt[i]) * up[i]);\n    orc_linear(gt, w->wd", "gt[i] = round_act(c, orc_silu(up[i]) * gt[i]);\n    orc_linear(gt, w->wd"),
 ("residual dropped after attention", "orc_linear(o, w->wo, NULL, QD, H, y);\n    for (int i = 0; i < H; ++i) x[i] += y[i];", "orc_linear(o, w->wo, NULL, QD, H, y);\n    for (int i = 0; i < H; ++i) x[i] = y[i];"),
 ("argmax: last index on ties", "if (x[i] > x[best]) best = i;", "if (x[i] >= x[best]) best = i;"),
 ("kv index: head and slot swapped", "return (((size_t)block * c->block_size + slot) * c->n_kv_heads + kvh) * c->head_dim;", "return (((size_t)block * c->n_kv_heads + kvh) * c->block_size + slot) * c->head_dim;"),
 ("bf16: truncation instead of nearest-even", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0u;"),
 ("bf16: ties away from zero", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0x8000u;"),
 ("query not rounded", "for (int i = 0; i < QD; ++i) q[i] = round_act(c, q[i]);", ";"),
 ("final norm uses no gain vector (g1 of nothing): head skips the norm", "orc_rmsnorm(x, w->gf, H, c->rms_eps, u);\n    for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);\n    orc_linear(u, w->wlm", "for (int i = 0; i < H; ++i) u[i] = round_act(c, x[i]);\n    orc_linear(u, w->wlm"),
 ("e4m3: ties away", "q = nearbyintf(a / ulp) * ulp;", "q = roundf(a / ulp) * ulp;"),
 ("e4m3: no saturation", "if (a > 448.0f) a = 448.0f;", ";"),
 ("e4m3: subnormal spacing", "q = nearbyintf(a * 512.0f) / 512.0f;", "q = nearbyintf(a * 1024.0f) / 1024.0f;"),
 ("philox: 9 rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
 ("philox: multipliers swapped", "(uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;", "(uint64_t)0xCD9E8D57u * c0, p1 = (uint64_t)0xD2511F53u * c2;"),
 ("uniform: 24 bits", "return ((float)(word >> 9) + 0.5f) * (1.0f / 8388608.0f);", "return ((float)(word >> 8) + 0.5f) * (1.0f / 16777216.0f);"),
 ("sample: Gumbel sign", "const float y = z - logf(-logf(u));\n        if (y > best) { second = best; best = y; best_i = i; }\n        else if (y > second) second = y;\n        if (z > zmax) zmax = z;", "const float y = z + logf(-logf(u));\n        if (y > best) { second = best; best = y; best_i = i; }\n        else if (y > second) second = y;\n        if (z > zmax) zmax = z;"),
 ("sample: temperature multiplies", "void orc_sample(const float *logits, int V, float temperature, uint64_t seed, uint32_t row, uint32_t pos,\n                int32_t *token, float *logprob, float *gap) {\n    const float inv_t = 1.0f / temperature;", "void orc_sample(const float *logits, int V, float temperature, uint64_t seed, uint32_t row, uint32_t pos,\n                int32_t *token, float *logprob, float *gap) {\n    const float inv_t = temperature;"),
 ("top-p: strict comparison at the cut", "if (cum >= (double)top_p) break;", "if (cum > (double)top_p + 1e-3) break;"),
 ("top-p: ties with the last kept entry dropped", "while (n < V && ord[n].z == ord[n - 1].z) ++n;", ";"),
 ("top-p: logprob under the full distribution", "*logprob = (float)((double)(logits[best_i] * inv_t) - ((double)zmax + log(mass)));", "*logprob = (float)((double)(logits[best_i] * inv_t) - ((double)zmax + log(sum)));"),
 ("full causal: future key visible", "for (int r = 0; r <= t; ++r) { /* causal mask: keys 0..t only */\n                    float dot = 0.0f;\n                    ORC_FOR_SUM(j, d)\n                        dot += Q[(size_t)t * QD + h * d + j] * Km[(size_t)r * KD + kvh * d + j];\n                    s[r] = dot * scale;\n                }\n                orc_softmax(s, t + 1, p);\n                for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;\n                ORC_FOR_SUM(r, t + 1)", "const int t2 = t + 1 < n ? t + 1 : t;\n                for (int r = 0; r <= t2; ++r) {\n                    float dot = 0.0f;\n                    ORC_FOR_SUM(j, d)\n                        dot += Q[(size_t)t * QD + h * d + j] * Km[(size_t)r * KD + kvh * d + j];\n                    s[r] = dot * scale;\n                }\n                orc_softmax(s, t2 + 1, p);\n                for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;\n                ORC_FOR_SUM(r, t2 + 1)"),
 ("full causal: last key not attended", "orc_softmax(s, t + 1, p);\n                for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;\n                ORC_FOR_SUM(r, t + 1)", "orc_softmax(s, t > 0 ? t : 1, p);\n                for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;\n                ORC_FOR_SUM(r, t > 0 ? t : 1)"),
]
CONTROL = ("control: the unchanged oracle passes its pins", None, None)


def mutant_verdict(item):
    """Plant one mistake in a scratch copy of its own, rebuild, run the pins; -> (name, verdict, first failing test)."""
    idx, (name, old, new) = item
    dst = tempfile.mkdtemp(prefix="oracle_mutant_%02d_" % idx)
    try:
        shutil.copytree(os.path.join(SRC, "oracle"), os.path.join(dst, "oracle"), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
        # of the tests only the oracle's pins and what they import
        shutil.copytree(os.path.join(SRC, "tests"), os.path.join(dst, "tests"),
                        ignore=lambda d, names: [n for n in names if not (n.startswith("test_oracle_") or n in ("util.py", "conftest.py", "golden")
                                                                          or d.endswith("golden")) or n == "test_oracle_mutations.py"])
        os.makedirs(os.path.join(dst, "paper_2511_00796_amd"))
        for f in ("__init__.py", "synth.py"):
            shutil.copy(os.path.join(SRC, "paper_2511_00796_amd", f), os.path.join(dst, "paper_2511_00796_amd", f))
        path = os.path.join(dst, "oracle", "decode_oracle.c")
        src = open(path).read()
        if old is not None:
            n = src.count(old)
            if n != 1 and not name.startswith("bf16"):
                return name, "PATTERN matches %d times" % n, ""
            open(path, "w").write(src.replace(old, new, 1))
        env = dict(os.environ, OMP_NUM_THREADS="2")
        r = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"], cwd=dst, capture_output=True, text=True, timeout=900, env=env)
        lines = [l for l in r.stdout.splitlines() if "FAILED" in l or "passed" in l or "failed" in l or "error" in l.lower()]
        first = next((l for l in lines if "FAILED" in l), lines[-1] if lines else "")
        failed = r.returncode == 1 and " failed" in r.stdout and " error" not in r.stdout.splitlines()[-1]
        return name, "caught" if failed else ("NOT CAUGHT" if r.returncode == 0 else "rc=%d: %s" % (r.returncode, r.stdout[-300:])), first[:110]
    finally:
        shutil.rmtree(dst, ignore_errors=True)


def run(select=None, workers=None, verbose=False):
    todo = [CONTROL] + [m for m in MUT if select is None or select in m[0]]
    workers = workers or max(1, min(8, (os.cpu_count() or 2) // 2))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        res = []
        for r in pool.map(mutant_verdict, enumerate(todo)):
            res.append(r)
            if verbose:
                print(r, flush=True)
    return res


def test_every_planted_mistake_in_the_oracle_fails_a_pin():
    res = run()
    assert res[0][1] == "NOT CAUGHT", res[0]             # the scratch copy works: the unchanged oracle passes
    missed = [r for r in res[1:] if r[1] != "caught"]
    print("caught %d of %d planted mistakes" % (len(res) - 1 - len(missed), len(res) - 1))
    assert len(res) - 1 == len(MUT) >= 34
    assert not missed, missed


if __name__ == "__main__":
    out = run(sys.argv[1] if len(sys.argv) > 1 else None, verbose=True)
    print("caught %d of %d" % (sum(1 for r in out[1:] if r[1] == "caught"), len(out) - 1))
    sys.exit(0 if out[0][1] == "NOT CAUGHT" and all(r[1] == "caught" for r in out[1:]) else 1)
