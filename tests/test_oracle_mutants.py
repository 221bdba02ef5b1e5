"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants one mistake in a COPY of oracle/cb_oracle.c (a dropped term, a
wrong sign or index, a transposed operand, a relaxed comparison), builds it on the
CPU, and runs tests/test_oracle_pins.py against that build in a child process:
the pins have to fail.  Nothing here touches the GPU or the HIP library.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cb_oracle.c")

MUTANTS = [
    # name, text in the oracle, replacement, expected number of occurrences
    ("non-strict threshold", "if (fabsf(d) > tau) ch = 1;", "if (fabsf(d) >= tau) ch = 1;", 2),
    ("no absolute value", "if (fabsf(d) > tau) ch = 1;", "if (d > tau) ch = 1;", 2),
    ("state never updated", "        if (m[p])\n            for (int c = 0; c < C; ++c) S[", "        if (0)\n            for (int c = 0; c < C; ++c) S[", 1),
    ("dilation offset sign", "int yi = yo * s - p + j, xi = xo * s - p + i;\n                    if (yi >= 0 && yi < H && xi >= 0 && xi < W && m[",
     "int yi = yo * s + p - j, xi = xo * s + p - i;\n                    if (yi >= 0 && yi < H && xi >= 0 && xi < W && m[", 1),
    ("dilation ignores stride", "int yi = yo * s - p + j, xi = xo * s - p + i;\n                    if (yi >= 0 && yi < H && xi >= 0 && xi < W && m[",
     "int yi = yo - p + j, xi = xo - p + i;\n                    if (yi >= 0 && yi < H && xi >= 0 && xi < W && m[", 1),
    ("transposed filter", "Ko[(c * kh + j) * kw + i]", "Ko[(c * kw + i) * kh + j]", 1),
    ("flipped filter (true convolution)", "int xi = xo * s - p + i;\n                if (xi < 0 || xi >= W) continue;",
     "int xi = xo * s - p + (kw - 1 - i);\n                if (xi < 0 || xi >= W) continue;", 1),
    ("dropped bias", "    double acc = b;\n", "    double acc = 0.0;\n", 1),
    ("wrong ReLU", "if (relu && acc < 0.0) acc = 0.0;", "if (relu && acc > 0.0) acc = 0.0;", 1),
    ("index list off by one", "if (mt[q]) idx[n++] = q;", "if (mt[q]) idx[n++] = q + 1;", 1),
    ("first frame not a full update", "    if (full)\n        memset(L->mt, 1, (size_t)Po);\n    else\n", "    if (0)\n        memset(L->mt, 1, (size_t)Po);\n    else\n", 1),
    ("updated outputs off by 1e-4 relative", "                    L->S, L->Kw, L->b, L->idx, L->N, vals);\n        for (int o = 0; o < L->O; ++o)\n            for (int q = 0; q < L->N; ++q)\n                L->OUT[(size_t)o * Po + L->idx[q]] = vals[(size_t)o * L->N + q];\n        free(vals);\n    }\n    return L->N;\n}\n\n/* One frame",
     "                    L->S, L->Kw, L->b, L->idx, L->N, vals);\n        for (int o = 0; o < L->O; ++o)\n            for (int q = 0; q < L->N; ++q)\n                L->OUT[(size_t)o * Po + L->idx[q]] = 1.0001f * vals[(size_t)o * L->N + q];\n        free(vals);\n    }\n    return L->N;\n}\n\n/* One frame", 1),
    ("bf16 truncation instead of nearest even", "double r = nearbyint(v / q) * q;", "double r = trunc(v / q) * q;", 1),
    ("floor-mode pooling", "int Hp = (Ho + w - 1) / w, Wp = (Wo + w - 1) / w;", "int Hp = Ho / w > 0 ? Ho / w : 1, Wp = Wo / w > 0 ? Wo / w : 1;", 2),
    ("pool takes the minimum", "if (v > best) best = v;", "if (v < best || best == -INFINITY) best = v;", 2),
    ("feed-forward keeps the old input", "    memcpy(S, x, (size_t)C * P * sizeof(float));\n    return M;", "    return M;", 1),
]


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new, count):
    src = open(SRC).read()
    assert src.count(old) == count, f"mutant '{name}' no longer matches the oracle source"
    mutated = tmp_path / "cb_oracle_mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libcb_oracle_mutant.so"
    subprocess.run(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib),
                    str(mutated), "-lm"], check=True)
    env = dict(os.environ, CB_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"the pins did not notice: {name}\n{r.stdout[-800:]}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()


def test_unmutated_oracle_passes_in_the_same_harness(tmp_path):
    lib = tmp_path / "libcb_oracle_same.so"
    subprocess.run(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib), SRC,
                    "-lm"], check=True)
    env = dict(os.environ, CB_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-800:]
