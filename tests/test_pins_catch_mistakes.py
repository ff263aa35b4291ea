"""The pins of the oracle must notice a plausible mistake anywhere in it (CPU only).

Each case plants one mistake in a copy of oracle/leann_oracle.c (a dropped term, a wrong sign or index, a swapped
operand, a changed rule), points the oracle binding at that copy and runs the oracle's pin tests in a fresh
interpreter: they have to fail.  The unmodified copy has to pass.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "leann_oracle.c")

MISTAKES = [
    # encoder
    ("enc", "segment embedding dropped", "te[i] + pe[i] + ew->seg[i]", "te[i] + pe[i]"),
    ("enc", "position embedding of t + 1", "*pe = ew->pos + (int64_t)t * d;", "*pe = ew->pos + (int64_t)(t + 1) * d;"),
    ("enc", "attention scale missing", "p[j] = s * scale;", "p[j] = s;"),
    ("enc", "query read from the key block", "const float *qi = qkv + (int64_t)i * 3 * d + h * dh;",
     "const float *qi = qkv + (int64_t)i * 3 * d + d + h * dh;"),
    ("enc", "values read from the key block", "2 * d + h * dh + c];", "d + h * dh + c];"),
    ("enc", "GELU argument scaled wrongly", "0.70710678118654752440f", "0.5f"),
    ("enc", "LayerNorm with the unbiased variance", "    var /= (float)d;\n    float inv", "    var /= (float)(d - 1);\n    float inv"),
    ("enc", "LayerNorm shift dropped", "float y = (row[i] - mean) * inv * g[i] + b[i];", "float y = (row[i] - mean) * inv * g[i];"),
    ("enc", "bias of the linear maps dropped", "y[(int64_t)t * out + o] = acc + b[o];", "y[(int64_t)t * out + o] = acc;"),
    ("enc", "weight rows mixed up", "*wr = W + (int64_t)o * in;", "*wr = W + (int64_t)(o % in) * in;"),
    ("enc", "softmax numerator shifted", "p[j] = expf(p[j] - mx);", "p[j] = expf(p[j] - mx) + 1e-3f;"),
    # PQ / ADC
    ("pq", "look-up table without the negation", "lut[m * ksub + c] = -s;", "lut[m * ksub + c] = s;"),
    ("pq", "shuffle draws modulo i instead of i + 1", "uint64_t j = splitmix64(&st) % (uint64_t)(i + 1);",
     "uint64_t j = splitmix64(&st) % (uint64_t)i;"),
    ("pq", "shuffle walks upwards", "for (int64_t i = n - 1; i >= 1; --i) {\n        uint64_t j = splitmix64(&st)",
     "for (int64_t i = 1; i <= n - 1; ++i) {\n        uint64_t j = splitmix64(&st)"),
    # search
    ("search", "ties broken towards the higher id", "return sa > sb || (sa == sb && ia < ib);",
     "return sa > sb || (sa == sb && ia > ib);"),
    ("search", "re-rank count rounded down", "ceilf(", "floorf("),
    ("search", "flush only when the exact queue is exhausted", "if (n_pend >= batch || (!has_unvisited && n_pend > 0)) {",
     "if ((!has_unvisited && n_pend > 0)) {"),
    ("search", "neighbour not marked as ADC-scored", "adc_seen[v] = 1;", "adc_seen[v] = 0;"),
    ("search", "selected candidate stays in the approximate queue", "aq[b] = aq[--n_aq];", "aq[b] = aq[n_aq - 1];"),
    ("search", "soft-delete filter switched off", "if (upd->deleted[eq[i].id]) eq[i].visited = -1;",
     "if (0 && upd->deleted[eq[i].id]) eq[i].visited = -1;"),
    # construction
    ("build", "RNG rule reversed", "if (simf(emb, d, ids[b], out[j]) > sim[b]) ok = 0;",
     "if (simf(emb, d, ids[b], out[j]) < sim[b]) ok = 0;"),
    ("build", "neighbours allowed one edge above the cap", "if (g.deg[r] <= M) continue;", "if (g.deg[r] <= M + 1) continue;"),
    ("build", "cap of the low-degree nodes ignored", "const int cap_v = (!is_hub || is_hub[v]) ? M : m;", "const int cap_v = M;"),
]
PIN_FILES = {"enc": ["tests/test_oracle_encoder.py"], "pq": ["tests/test_oracle_pq.py"],
             "search": ["tests/test_oracle_search.py"], "build": ["tests/test_oracle_build.py"]}


def run_pins(src_path, files):
    env = dict(os.environ, LEANN_ORACLE_SRC=src_path)
    return subprocess.run([sys.executable, "-m", "pytest", *files, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True)


def test_unmodified_copy_passes(tmp_path):
    copy = tmp_path / "leann_oracle.c"
    copy.write_text(open(SRC).read())
    p = run_pins(str(copy), sum(PIN_FILES.values(), []))
    assert p.returncode == 0, p.stdout[-2000:]


@pytest.mark.parametrize("part,name,old,new", MISTAKES, ids=[m[1] for m in MISTAKES])
def test_planted_mistake_is_noticed(tmp_path, part, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"pattern for '{name}' no longer in the oracle: update this test"
    copy = tmp_path / "leann_oracle.c"
    copy.write_text(text.replace(old, new, 1))
    p = run_pins(str(copy), PIN_FILES[part])
    assert p.returncode != 0, f"'{name}' went unnoticed by {PIN_FILES[part]}"
