"""Checks that the oracle's pins have teeth: each plausible mistake planted in a
copy of the C oracle (CPU only, in a temporary directory) must make the pin
suite fail.  The real oracle is never modified."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in rocket_oracle.c, replacement)
MUTATIONS = [
    ("tap index without padding offset", "(i64)t + (i64)j * dil - pad;\n            if (idx >= 0 && idx < L)\n                acc +=",
     "(i64)t + (i64)j * dil;\n            if (idx >= 0 && idx < L)\n                acc +="),
    ("flipped kernel", "acc += (double)w[c * len + j] * (double)row[idx];", "acc += (double)w[c * len + (len - 1 - j)] * (double)row[idx];"),
    ("dilation ignored", "(i64)t + (i64)j * dil - pad;\n            if (idx >= 0 && idx < L)\n                acc +=",
     "(i64)t + (i64)j - pad;\n            if (idx >= 0 && idx < L)\n                acc +="),
    ("wrong channel gather", "const float *row = x + (size_t)ch[c] * (size_t)L;\n        for (int j = 0; j < len; ++j) {\n            i64 idx = (i64)t",
     "const float *row = x + (size_t)c * (size_t)L;\n        for (int j = 0; j < len; ++j) {\n            i64 idx = (i64)t"),
    ("bias dropped", "return acc + bias;", "return acc;"),
    ("output length off by one", "return L + 2 * pad - (len - 1) * dil;", "return L + 2 * pad - (len - 1) * dil - 1;"),
    ("non-strict Heaviside", "if (y > 0.0) ++cnt;", "if (y >= 0.0) ++cnt;"),
    ("shift sign", "soft += 1.0 / (1.0 + exp(-(lambda * y + shift)));", "soft += 1.0 / (1.0 + exp(-(lambda * y - shift)));"),
    ("lambda dropped in forward", "soft += 1.0 / (1.0 + exp(-(lambda * y + shift)));", "soft += 1.0 / (1.0 + exp(-(y + shift)));"),
    ("softPPV not averaged", "osoft[o] = soft / (double)n;", "osoft[o] = soft;"),
    ("gradient without 1/n", "double q = gs * (lambda / (double)n) * sg * (1.0 - sg);", "double q = gs * lambda * sg * (1.0 - sg);"),
    ("gradient without s(1-s)", "double q = gs * (lambda / (double)n) * sg * (1.0 - sg);", "double q = gs * (lambda / (double)n) * sg;"),
    ("weight gradient at the wrong tap", "if (idx >= 0 && idx < L) gw[c * len + j] += q * (double)row[idx];",
     "if (idx >= 0 && idx < L) gw[c * len + (len - 1 - j)] += q * (double)row[idx];"),
    ("batch sum lost", "grad_b[k] += q;", "grad_b[k] = q;"),
    ("max sub-gradient at the last position", "if (y > best) { best = y; arg = t; }\n                double sg", "if (y >= best) { best = y; arg = n - 1; }\n                double sg"),
]


@pytest.fixture(scope="module")
def clean_copy(tmp_path_factory):
    base = tmp_path_factory.mktemp("oracle_mutants")
    return str(base)


def _run_pins(workdir):
    env = dict(os.environ, PYTHONPATH=workdir + os.pathsep + ROOT)
    tests = [os.path.join(ROOT, "tests", "test_oracle_pins.py")]
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           "--rootdir", workdir, "-c", os.devnull] + tests,
                          env=env, cwd=workdir, capture_output=True, text=True, timeout=600)


def _make_copy(workdir, name, old=None, new=None):
    d = os.path.join(workdir, name)
    os.makedirs(d)
    pkg = os.path.join(d, "oracle")
    shutil.copytree(os.path.join(ROOT, "oracle"), pkg, ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copy(os.path.join(ROOT, "tests", "conftest.py"), os.path.join(d, "conftest.py"))
    if old is not None:
        path = os.path.join(pkg, "rocket_oracle.c")
        src = open(path).read()
        assert src.count(old) >= 1, "mutation target not found: " + old[:40]
        open(path, "w").write(src.replace(old, new, 1))
    return d


def test_unmutated_copy_passes(clean_copy):
    r = _run_pins(_make_copy(clean_copy, "clean"))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(clean_copy, idx):
    name, old, new = MUTATIONS[idx]
    r = _run_pins(_make_copy(clean_copy, "m%d" % idx, old, new))
    assert r.returncode != 0, "pins did not notice: " + name
    # it must be a failing pin, not a mutant that does not compile or import
    assert " failed" in r.stdout and "CalledProcessError" not in r.stdout and "ImportError" not in r.stdout, r.stdout[-800:]
