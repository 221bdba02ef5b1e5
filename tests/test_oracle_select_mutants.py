"""The pins of the threshold-selection oracle must notice a plausible mistake in it.

Each case plants one mistake in a COPY of oracle/cb_select.py and runs tests/test_oracle_select.py
against that copy in a child process: the pins have to fail.  No GPU.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cb_select.py")

MUTANTS = [
    ("limit not strict", "            if loss > max_loss[l]:", "            if loss >= max_loss[l]:"),
    ("keeps the value that exceeded the limit", "            if loss > max_loss[l]:\n                break\n            kept = tau\n",
     "            kept = tau\n            if loss > max_loss[l]:\n                break\n"),
    ("loss measured against the all-zero network", "        base = quality(net, sequences, refs, taus)",
     "        base = quality(net, sequences, refs, [0.0] * n)"),
    ("threshold sequence in float64", "            tau = np.float32(tau * np.float32(factor))", "            tau = float(tau) * factor"),
    ("absolute instead of squared differences", "        total += float(np.sum(d * d))", "        total += float(np.sum(np.abs(d)))"),
    ("sequences not played from a reset chain", "    for seq, ref in zip(sequences, refs):\n        net.reset()\n",
     "    for seq, ref in zip(sequences, refs):\n"),
    ("reference taken at the first frame", "        for f in seq:\n            out = net.forward(f, zeros)\n        refs.append",
     "        for f in seq[:1]:\n            out = net.forward(f, zeros)\n        refs.append"),
    ("later layers not at zero", "    taus = [np.float32(0.0)] * n", "    taus = [np.float32(tau0)] * n"),
    ("sum instead of mean", "    return total / count", "    return total"),
    ("pooling skipped", "            if self.pool_after[l]:\n                orc.pool_update", "            if False:\n                orc.pool_update"),
]


def _run(env):
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_select.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutant '{name}' no longer matches the oracle source"
    mutated = tmp_path / "cb_select_mutant.py"
    mutated.write_text(src.replace(old, new))
    r = _run(dict(os.environ, CB_SELECT_SRC=str(mutated)))
    assert r.returncode != 0, f"the pins did not notice: {name}\n{r.stdout[-800:]}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()


def test_unmutated_copy_passes_in_the_same_harness(tmp_path):
    same = tmp_path / "cb_select_same.py"
    same.write_text(open(SRC).read())
    r = _run(dict(os.environ, CB_SELECT_SRC=str(same)))
    assert r.returncode == 0, r.stdout[-800:]
