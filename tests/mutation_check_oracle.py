"""Mutation check of the oracle's pins (CPU only; run by hand: python tests/mutation_check_oracle.py).

Plants one plausible mistake at a time (a wrong comparison, a dropped term, a shifted index, a
transposed head mapping) in a temporary COPY of oracle/specpv_oracle.c and runs
tests/test_oracle_pins.py against that copy: every planted mistake has to make a pin fail.
Nothing here touches the repository's oracle, the GPU path or a GPU."""
import os
import shutil
import subprocess
import sys
import tempfile
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MUT = [
 ("if (x > mx) mx = x;", "if (x >= mx + 1e300) mx = x;", "kmax never updated"),
 ("if (x < mn) mn = x;", "if (x > mn) mn = x;", "kmin takes max"),
 ("int t1 = (i + 1) * B < L ? (i + 1) * B : L;", "int t1 = (i + 1) * B < L ? (i + 1) * B - 1 : L;", "block one token short"),
 ("= da > db ? da : db;", "= da < db ? da : db;", "eq2 min instead of max"),
 ("db += q[d] * b[d];", "db += q[d] * a[d];", "eq2 ignores kmin"),
 ("int h = g * G + hh;\n                    const double *q = Q + ((size_t)j * Hq + h) * D;\n                    const double *a = kmax + ((size_t)i * Hkv + g) * D;\n                    const double *b = kmin + ((size_t)i * Hkv + g) * D;\n                    double da", "int h = hh * Hkv + g;\n                    const double *q = Q + ((size_t)j * Hq + h) * D;\n                    const double *a = kmax + ((size_t)i * Hkv + g) * D;\n                    const double *b = kmin + ((size_t)i * Hkv + g) * D;\n                    double da", "GQA head mapping interleaved"),
 ("sum += pa > pb ? pa : pb;", "sum += pa < pb ? pa : pb;", "channel bound min"),
 ("out = acc / (double)R;", "out = acc / (double)M;", "mean over M"),
 ("if (row[r] > out) out = row[r];", "if (row[r] < out) out = row[r];", "max reducer is min"),
 ("acc += row[(size_t)last_node * G + hh];", "acc += row[(size_t)hh * M + last_node];", "last reducer wrong rows"),
 ("for (int i = nb - nr; i < nb; ++i) keep[i] = 1;", "for (int i = nb - nr + 1; i < nb; ++i) keep[i] = 1;", "one recent block short"),
 ("if (best < 0 || si > best_s)", "if (best < 0 || si >= best_s)", "ties to higher index"),
 ("float si = (float)scores[(size_t)g * nb + i];", "double si = scores[(size_t)g * nb + i];", "no fp32 rounding in compare"),
 ("for (int i = 0; i < ns; ++i) keep[i] = 1;", "for (int i = 0; i < ns - 1; ++i) keep[i] = 1;", "one sink block short"),
 ("double scale = 1.0 / sqrt((double)D);", "double scale = 1.0 / (double)D;", "scale 1/D"),
 ("for (int a = j; a >= 0; a = parent[a]) anc[a] = 1;", "for (int a = parent[j]; a >= 0; a = parent[a]) anc[a] = 1;", "node does not see itself"),
 ("for (int a = j; a >= 0; a = parent[a]) anc[a] = 1;", "for (int a = 0; a <= j; ++a) anc[a] = 1;", "causal instead of tree mask"),
 ("if (!keep[t / B]) continue;", "if (!keep[t / B] && t / B != 0) continue;", "block 0 always attended"),
 ("vp[n] = Vd + ((size_t)a * Hkv + g) * D;", "vp[n] = Vd + ((size_t)j * Hkv + g) * D;", "draft V of the query node"),
 ("int g = h / G;", "int g = h % Hkv;", "attention GQA mapping interleaved"),
 ("lse[(size_t)j * Hq + h] = zmax + log(denom);", "lse[(size_t)j * Hq + h] = log(denom);", "lse without max"),
 ("const double *kk = K + ((size_t)t * Hkv + g) * D;", "const double *kk = K + ((size_t)t * Hkv + g) * D + 0; if (t == L - 1) continue;", "last token dropped"),
]
src = open(os.path.join(ROOT, "oracle/specpv_oracle.c")).read()
res = []
for old, new, what in MUT:
    if src.count(old) < 1:
        res.append((what, "PATTERN NOT FOUND")); continue
    d = os.path.join(tempfile.gettempdir(), "specpv_oracle_mutant_%d" % os.getpid())
    shutil.rmtree(d, ignore_errors=True)
    os.makedirs(d)
    for x in ("oracle", "tests", "workloads.py", "paper_2512_02337_amd", "include"):
        s = os.path.join(ROOT, x)
        (shutil.copytree if os.path.isdir(s) else shutil.copy)(s, os.path.join(d, x), **({"ignore": shutil.ignore_patterns("_build", "__pycache__", "*.so.tmp*")} if os.path.isdir(s) else {}))
    os.remove(os.path.join(d, "oracle/libspecpv_oracle.so"))
    open(os.path.join(d, "oracle/specpv_oracle.c"), "w").write(src.replace(old, new, 1))
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"], cwd=d, capture_output=True, text=True)
    tail = [l for l in r.stdout.splitlines() if l.startswith("FAILED") or "passed" in l or "failed" in l]
    res.append((what, "caught: " + tail[0][:110] if r.returncode != 0 and tail else ("NOT CAUGHT" if r.returncode == 0 else "error " + r.stdout[-300:])))
    shutil.rmtree(d, ignore_errors=True)
    print("%-45s %s" % res[-1], flush=True)
missed = [w for w, r in res if not r.startswith("caught")]
print("%d of %d planted mistakes caught" % (len(res) - len(missed), len(res)))
sys.exit(1 if missed else 0)
