"""How strong are the oracle's pins?  Each case plants one plausible mistake in a copy of the oracle's C
source (a dropped term, a wrong index, a reversed comparison, a missing factor), builds the copy on the
CPU and runs tests/test_oracle_pins.py against it in a child process: the pins must fail.  The unmodified
source must pass the same way.  Nothing here touches the GPU."""
import os
import subprocess
import sys

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in oracle/pqc_oracle.c, replacement); every text must occur exactly once in the source
MUTATIONS = [
    ("scores: only the group's last head", "a32 = (h == 0) ? qv : a32 + qv;\n        a64 += (double)qv;",
     "a32 = qv;\n        a64 = (double)qv;"),
    ("scores: every partition reads partition 0's centroids", "centroids + (((int64_t)u * M + j) * C + code) * Dm;",
     "centroids + (((int64_t)u * M + 0) * C + code) * Dm;"),
    ("scores: query dimensions interleaved instead of blocked",
     "p32 = fmaf(qs32[j * Dm + e], cv[e], p32);\n          p64 += qs64[j * Dm + e] * (double)cv[e];",
     "p32 = fmaf(qs32[e * M + j], cv[e], p32);\n          p64 += qs64[e * M + j] * (double)cv[e];"),
    ("scores: partitions overwrite instead of adding", "s32 = (j == 0) ? p32 : s32 + p32;\n        s64 += p64;",
     "s32 = p32;\n        s64 = p64;"),
    ("scores: code of the neighbouring token", "int code = codes[((int64_t)u * N + t) * M + j];",
     "int code = codes[((int64_t)u * N + (t + 1 < N ? t + 1 : t)) * M + j];"),
    ("select: smallest scores first", "if (x->s > y->s) return -1;\n  if (x->s < y->s) return 1;",
     "if (x->s > y->s) return 1;\n  if (x->s < y->s) return -1;"),
    ("select: ties go to the higher index", "return (x->t > y->t) - (x->t < y->t);", "return (x->t < y->t) - (x->t > y->t);"),
    ("select: scores read from the start of the array", "arr[t].s = score[(int64_t)u * N + I + t];",
     "arr[t].s = score[(int64_t)u * N + t];"),
    ("select: local window one token early", "o[I + K + t] = (int32_t)(N - L + t);", "o[I + K + t] = (int32_t)(N - L + t - 1);"),
    ("attention: softmax scale dropped", "logit[i] = scale * s;", "logit[i] = s;"),
    ("attention: keys where values belong", "acc += logit[i] * (double)elem(v, dtype, (u * N + t) * D + d);",
     "acc += logit[i] * (double)elem(k, dtype, (u * N + t) * D + d);"),
    ("attention: not normalised", "out[(int64_t)bh * D + d] = acc / den;", "out[(int64_t)bh * D + d] = acc;"),
    ("attention: wrong KV head for a query head", "int b = bh / Hq, h = bh % Hq, g = h / G;", "int b = bh / Hq, h = bh % Hq, g = h % Hkv;"),
    ("bf16 widened with the wrong shift", "(uint32_t)((const uint16_t*)base)[i] << 16;", "(uint32_t)((const uint16_t*)base)[i] << 15;"),
    ("k-means: mean over one member too many", "(float)(sum[a * dm + e] / (double)cnt[a]);", "(float)(sum[a * dm + e] / (double)(cnt[a] + 1));"),
    ("k-means: ties go to the higher centroid", "      if (d2 < best) {\n        best = d2;\n        arg = a;\n      }\n    }\n    codes[t] = (uint8_t)arg;",
     "      if (d2 <= best) {\n        best = d2;\n        arg = a;\n      }\n    }\n    codes[t] = (uint8_t)arg;"),
    ("k-means: distance without the square", "        d2 += diff * diff;\n      }\n      if (d2 < best) {\n        best = d2;\n        arg = a;\n      }\n    }\n    codes[t]",
     "        d2 += diff < 0 ? -diff : diff;\n      }\n      if (d2 < best) {\n        best = d2;\n        arg = a;\n      }\n    }\n    codes[t]"),
    ("appended token: nearest by the first partition's centroids", "(double)centroids[(((int64_t)u * M + j) * C + a) * Dm + e];",
     "(double)centroids[(((int64_t)u * M + 0) * C + a) * Dm + e];"),
    ("block counts: block of the next token", "counts[u * nb + t / block] += 1;", "counts[u * nb + (t + 1 < N ? t + 1 : t) / block] += 1;"),
    ("block ranking: ties go to the higher block", "(best < 0 || c[j] > c[best])", "(best < 0 || c[j] >= c[best])"),
]


def _run_pins(lib_path):
    env = dict(os.environ, PQC_ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def _build_variant(tmp_path, source_text, tag):
    src, lib = tmp_path / f"oracle_{tag}.c", tmp_path / f"liboracle_{tag}.so"
    src.write_text(source_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fopenmp-simd", "-ffp-contract=off", "-mavx2", "-mfma", "-shared", "-fPIC",
                    str(src), "-o", str(lib), "-lm"], check=True)
    return str(lib)


def test_unmodified_copy_passes_the_pins(tmp_path):
    r = _run_pins(_build_variant(tmp_path, open(oracle_build.SRC).read(), "same"))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_the_pins(tmp_path, name, old, new):
    text = open(oracle_build.SRC).read()
    assert text.count(old) == 1, f"the oracle's source no longer holds this text exactly once: {old!r}"
    r = _run_pins(_build_variant(tmp_path, text.replace(old, new), "mutant"))
    assert r.returncode != 0, f"no pin noticed: {name}"
    assert " failed" in r.stdout, r.stdout[-1500:]  # a failing pin, not a crash of the child process
