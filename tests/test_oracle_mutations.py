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


# (name, oracle file, pin file, text, replacement): mistakes in the Python parts of the oracle
PY_MUTATIONS = [
    ("z-score with the sample std", "prologue.py", "test_oracle_prologue.py",
     "std = np.sqrt(((v - mean) ** 2).mean(axis=-1, keepdims=True))",
     "std = np.sqrt(((v - mean) ** 2).sum(axis=-1, keepdims=True) / (v.shape[-1] - 1))"),
    ("z-score without centring", "prologue.py", "test_oracle_prologue.py",
     "z = np.where(std > 0, (v - mean) / np.where(std > 0, std, 1.0), 0.0)",
     "z = np.where(std > 0, v / np.where(std > 0, std, 1.0), 0.0)"),
    ("constant row not zeroed", "prologue.py", "test_oracle_prologue.py",
     "z = np.where(std > 0, (v - mean) / np.where(std > 0, std, 1.0), 0.0)",
     "z = (v - mean) / np.where(std > 0, std, 1.0) + (std == 0)"),
    ("ridge intercept penalised", "ridge.py", "test_oracle_ridge.py",
     "return w, y_mean - x_mean @ w", "return w, (y_mean - x_mean @ w) / (1.0 + alpha / n)"),
    ("ridge penalty dropped in the dual branch", "ridge.py", "test_oracle_ridge.py",
     "Xc @ Xc.T + alpha * np.eye(n)", "Xc @ Xc.T + 1e-9 * np.eye(n)"),
    ("ridge columns not centred", "ridge.py", "test_oracle_ridge.py", "Xc = X - x_mean", "Xc = X"),
    ("ridge penalty squared", "ridge.py", "test_oracle_ridge.py",
     "Xc.T @ Xc + alpha * np.eye(p)", "Xc.T @ Xc + alpha * alpha * np.eye(p)"),
    ("loss gradient without 2/B", "train.py", "test_oracle_train.py",
     "(2.0 / len(y)) * r[:, None] * coef[None, :]", "r[:, None] * coef[None, :]"),
    ("update with the wrong sign", "train.py", "test_oracle_train.py",
     "np.asarray(kr[\"weights\"], np.float64) - float(lr)", "np.asarray(kr[\"weights\"], np.float64) + float(lr)"),
    ("bias not updated", "train.py", "test_oracle_train.py",
     "b = np.asarray(kr[\"bias\"], np.float64) - float(lr) * np.asarray(gb, np.float64)",
     "b = np.asarray(kr[\"bias\"], np.float64)"),
    ("re-centring over the whole kernel", "train.py", "test_oracle_train.py",
     "                row = w[lo + c * ln: lo + (c + 1) * ln]\n                row -= row.mean()",
     "                row = w[lo + c * ln: lo + (c + 1) * ln]\n                row -= w[lo: lo + ln * int(kr[\"n_ch\"][k])].mean()"),
    ("max plane left out of the step", "train.py", "test_oracle_train.py",
     "g_max = G[:, :K] if mask & 1 else None", "g_max = None"),
    ("soft plane taken from the wrong columns", "train.py", "test_oracle_train.py",
     "g_soft = G[:, (planes - 1) * K:]", "g_soft = G[:, :K]"),
    ("two-valued weights that do not sum to zero", "minirocket.py", "test_oracle_minirocket.py",
     "LOW, HIGH = -1.0, 2.0", "LOW, HIGH = -1.0, 3.0"),
    ("weight set in the wrong order", "minirocket.py", "test_oracle_minirocket.py",
     "SET = list(itertools.combinations(range(LENGTH), 3))", "SET = list(itertools.combinations(range(LENGTH), 3))[::-1]"),
    ("pairs instead of triples", "minirocket.py", "test_oracle_minirocket.py",
     "SET = list(itertools.combinations(range(LENGTH), 3))", "SET = list(itertools.combinations(range(LENGTH), 2)) * 3"),
    ("additions with the wrong multiple", "minirocket.py", "test_oracle_minirocket.py",
     "return 3.0 * high - sum(taps)", "return 2.0 * high - sum(taps)"),
    ("additions without the padding", "minirocket.py", "test_oracle_minirocket.py",
     "total[p:p + L] = x[ch].sum(axis=0)", "total[:L] = x[ch].sum(axis=0)"),
    ("additions on the first channel only", "minirocket.py", "test_oracle_minirocket.py",
     "total[p:p + L] = x[ch].sum(axis=0)", "total[p:p + L] = x[ch[0]]"),
    ("bias with the wrong sign", "minirocket.py", "test_oracle_minirocket.py",
     "bias[k] = np.float32(-np.partition(y, rank[k])[rank[k]])", "bias[k] = np.float32(np.partition(y, rank[k])[rank[k]])"),
    ("rank counted from the top", "minirocket.py", "test_oracle_minirocket.py",
     "bias[k] = np.float32(-np.partition(y, rank[k])[rank[k]])",
     "bias[k] = np.float32(-np.partition(y, len(y) - 1 - rank[k])[len(y) - 1 - rank[k]])"),
    ("rank from q n instead of q (n - 1)", "minirocket.py", "test_oracle_minirocket.py",
     "rank[k] = int(math.floor(q[k] * (len(y) - 1)))", "rank[k] = min(len(y) - 1, int(math.floor(q[k] * len(y))) + 1)"),
    ("bias taken from the first example always", "minirocket.py", "test_oracle_minirocket.py",
     "y = output_by_additions(x_train[ex[k]], kr, k)", "y = output_by_additions(x_train[0], kr, k)"),
    ("group dilation beyond the series", "minirocket.py", "test_oracle_minirocket.py",
     "d = max(1, min(d, (L - 1) // (LENGTH - 1)))", "d = max(1, 2 * d)"),
]


@pytest.fixture(scope="module")
def clean_copy(tmp_path_factory):
    base = tmp_path_factory.mktemp("oracle_mutants")
    return str(base)


def _run_pins(workdir, pin_file="test_oracle_pins.py"):
    env = dict(os.environ, PYTHONPATH=workdir + os.pathsep + ROOT)
    tests = [os.path.join(ROOT, "tests", pin_file)]
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           "--rootdir", workdir, "-c", os.devnull] + tests,
                          env=env, cwd=workdir, capture_output=True, text=True, timeout=600)


def _make_copy(workdir, name, old=None, new=None, target="rocket_oracle.c"):
    d = os.path.join(workdir, name)
    os.makedirs(d)
    pkg = os.path.join(d, "oracle")
    # a mutant of the C file must rebuild its library; the others can take the built one along
    skip = ("*.so", "__pycache__") if target.endswith(".c") else ("__pycache__",)
    shutil.copytree(os.path.join(ROOT, "oracle"), pkg, ignore=shutil.ignore_patterns(*skip))
    shutil.copy(os.path.join(ROOT, "tests", "conftest.py"), os.path.join(d, "conftest.py"))
    if old is not None:
        path = os.path.join(pkg, target)
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


@pytest.mark.parametrize("idx", range(len(PY_MUTATIONS)), ids=[m[0] for m in PY_MUTATIONS])
def test_planted_mistake_in_the_python_parts_is_caught(clean_copy, idx):
    name, target, pin_file, old, new = PY_MUTATIONS[idx]
    r = _run_pins(_make_copy(clean_copy, "p%d" % idx, old, new, target), pin_file)
    assert r.returncode != 0, "pins did not notice: " + name
    assert " failed" in r.stdout and "CalledProcessError" not in r.stdout and "ImportError" not in r.stdout, r.stdout[-800:]
