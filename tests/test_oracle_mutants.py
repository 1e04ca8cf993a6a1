"""Do the oracle's pins bite?  Each case plants ONE plausible mistake in a
scratch copy of the oracle (a wrong sign, divisor, index, order ...) and runs
the CPU pins on that copy in a separate interpreter: the pins must fail.  The
unmodified copy must pass, so a failure is due to the planted mistake and not
to the copying.  Nothing here touches the GPU library or the real oracle."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_partition.py", "test_oracle_step.py", "test_oracle_opt.py", "test_oracle_pattern.py"]

# (file inside oracle/, text as it stands, text with the mistake)
MUTANTS = {
    "sign of the local update": ("ds_oracle.c", "acc += x - lrd * g;", "acc += x + lrd * g;"),
    "gradient term dropped": ("ds_oracle.c", "acc += x - lrd * g;", "acc += x;"),
    "divisor of the group mean": ("ds_oracle.c", "const float m = (float)(acc / (double)n);\n            for (int32_t q = 0; q < n; ++q) X[",
                                  "const float m = (float)(acc / (double)(n + 1));\n            for (int32_t q = 0; q < n; ++q) X["),
    "divisor of the column mean": ("ds_oracle.c", "xbar[p] = s / (double)W;", "xbar[p] = s / (double)(W - 1);"),
    "absolute value for the square": ("ds_oracle.c", "s += e * e;", "s += fabs(e);"),
    "modulo for multiply-high": ("ds_oracle.c", "int32_t j = (int32_t)(uint64_t)(wide >> 64);", "int32_t j = (int32_t)(r % (uint64_t)(i + 1)); (void)wide;"),
    "iteration t for t+1 in the key": ("ds_oracle.c", "(t + 1) * gamma", "t * gamma"),
    "momentum applied to the gradient": ("ds_oracle.c", "v = mud * (double)V[i * ldv + p] + d;", "v = (double)V[i * ldv + p] + mud * d;"),
    "sign of the weight decay": ("ds_oracle.c", "const double d = g + wdd * x;", "const double d = g - wdd * x;"),
    "SWA factor on the wrong term": ("ds_oracle.c", "(float)(fd * (double)S[i * lds + p] + (1.0 - fd) * (double)m)", "(float)((1.0 - fd) * (double)S[i * lds + p] + fd * (double)m)"),
    "order of the mixing-matrix product": ("mixing.py", "acc = Wk @ acc", "acc = acc @ Wk"),
    "mixing weight 1/N for 1/|group|": ("mixing.py", "Wk[i, j] = 1.0 / len(members)", "Wk[i, j] = 1.0 / N"),
    "representative does not rotate": ("pattern.py", "rep = [e[t % len(e)] for e in eligible]", "rep = [e[0] for e in eligible]"),
}


def scratch_copy(dst):
    os.makedirs(os.path.join(dst, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(dst, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(dst, "tests", "golden"))
    for name in PINS + ["conftest.py"]:
        shutil.copy(os.path.join(ROOT, "tests", name), os.path.join(dst, "tests", name))


def run_pins(repo):
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join("tests", n) for n in PINS]
    return subprocess.run(cmd, cwd=repo, env=env, capture_output=True, text=True, timeout=600)


def test_the_unmodified_copy_passes_its_pins(tmp_path):
    repo = str(tmp_path / "copy")
    scratch_copy(repo)
    res = run_pins(repo)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_a_planted_mistake_fails_the_pins(tmp_path, name):
    fname, good, bad = MUTANTS[name]
    repo = str(tmp_path / "mutant")
    scratch_copy(repo)
    path = os.path.join(repo, "oracle", fname)
    text = open(path).read()
    assert good in text, "the oracle no longer contains the line this mistake is planted in"
    with open(path, "w") as fh:
        fh.write(text.replace(good, bad, 1))
    res = run_pins(repo)
    assert res.returncode != 0, "the pins did not notice: " + name
    assert "failed" in res.stdout or "error" in res.stdout.lower(), res.stdout[-1500:]
