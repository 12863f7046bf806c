"""Two CPU checks of the oracle as test infrastructure:

* planted mistakes -- every mutant of oracle/bnn_oracle.c or of the Python composition in
  oracle/__init__.py (a wrong comparison, sign, index, pad value, pool order, flatten order, ...)
  must make at least one pin of tests/test_oracle_pins.py fail;
* the pins run once more against an AddressSanitizer + UndefinedBehaviorSanitizer build of the
  C oracle (gcc), in a fresh process.

Each run happens in a scratch copy of oracle/, workloads/ and the pin tests; nothing in the
repository is modified.  The stored regression logits are excluded from those runs: they were
written by the oracle and pin nothing.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C_FILE = os.path.join("oracle", "bnn_oracle.c")
PY_FILE = os.path.join("oracle", "__init__.py")

# (name, file, text to find, replacement)
MUTANTS = [
    ("step uses >= instead of >", C_FILE,
     "int above = x[r * c + ch] > thr[ch];", "int above = x[r * c + ch] >= thr[ch];"),
    ("step ignores the flip flag", C_FILE,
     "out[r * c + ch] = (above != f) ? 1 : -1;", "out[r * c + ch] = above ? 1 : -1;"),
    ("conv taps mirrored vertically", C_FILE,
     "const int yy = y + i - pad;", "const int yy = y - i + pad;"),
    ("conv column offset uses the row tap", C_FILE,
     "const int xx = x + j - pad;", "const int xx = x + i - pad;"),
    ("conv pads with 0", C_FILE, "a = pad_value;", "a = 0;"),
    ("conv weight taps transposed", C_FILE,
     "wt[(((size_t)o * kh + i) * kw + j) * c_in + c];", "wt[(((size_t)o * kh + j) * kw + i) * c_in + c];"),
    ("conv drops the last input channel", C_FILE,
     "for (int c = 0; c < c_in; ++c) {", "for (int c = 0; c < c_in - (c_in > 1); ++c) {"),
    ("fc weight matrix transposed", C_FILE, "(int32_t)wt[o * k + t];", "(int32_t)wt[(t * n + o) % (n * k)];"),
    ("fc subtracts instead of adding", C_FILE,
     "sum += (int32_t)a[r * k + t] * (int32_t)wt[o * k + t];", "sum -= (int32_t)a[r * k + t] * (int32_t)wt[o * k + t];"),
    ("dot skips the first element", C_FILE,
     "for (int64_t t = 0; t < k; ++t) sum += (int32_t)a[t] * (int32_t)b[t];",
     "for (int64_t t = (k > 1); t < k; ++t) sum += (int32_t)a[t] * (int32_t)b[t];"),
    ("pool takes the minimum", C_FILE, "if (v > best) best = v;", "if (v < best) best = v;"),
    ("pool window column uses the row index", C_FILE, "2 * xx + j) * c + ch];", "2 * xx + i) * c + ch];"),
    ("model: binary conv padded with 0", PY_FILE,
     "pre4 = conv2d(act, L.weights, 1, -1)", "pre4 = conv2d(act, L.weights, 1, 0)"),
    ("model: first layer ignores its pad value", PY_FILE,
     "pre4 = conv2d(act, L.weights, L.pad, first_pad_value)", "pre4 = conv2d(act, L.weights, L.pad, -1)"),
    ("model: pool order swapped", PY_FILE,
     "if L.pool == 2 and pool_first:", "if L.pool == 2 and not pool_first:"),
    ("model: flatten in (c, h, w) order", PY_FILE,
     "a = act.reshape(act.shape[0], -1) ", "a = (act.transpose(0, 3, 1, 2) if act.ndim == 4 else act).reshape(act.shape[0], -1) "),
    ("model: step applied before the pool in both orders", PY_FILE,
     "s = step(maxpool2(pre4), L.thr, L.flip)", "s = maxpool2(step(pre4, L.thr, L.flip))"),
]


def scratch_tree(tmp_path):
    for d in ("oracle", "workloads"):
        shutil.copytree(os.path.join(ROOT, d), tmp_path / d,
                        ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    os.makedirs(tmp_path / "tests")
    for f in ("__init__.py", "conftest.py", "helpers.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), tmp_path / "tests" / f)
    return tmp_path


def run_pins(tree, env_extra=None, stop_at_first=True):
    env = dict(os.environ)
    env.pop("PYTHONPATH", None)
    env.update(env_extra or {})
    cmd = [sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-q", "-k", "not golden",
           "-p", "no:cacheprovider"] + (["-x"] if stop_at_first else [])
    return subprocess.run(cmd, cwd=tree, env=env, capture_output=True, text=True, timeout=600)


def test_pins_pass_on_the_unmodified_copy(tmp_path):
    r = run_pins(scratch_tree(tmp_path))
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]


@pytest.mark.parametrize("name,rel,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(tmp_path, name, rel, old, new):
    tree = scratch_tree(tmp_path)
    path = tree / rel
    text = path.read_text()
    assert text.count(old) >= 1, f"mutant '{name}' no longer applies: its source line changed"
    path.write_text(text.replace(old, new))
    r = run_pins(tree)
    assert r.returncode != 0, f"no pin notices: {name}"
    assert " failed" in r.stdout or " error" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


def test_pins_under_address_and_undefined_sanitizers(tmp_path):
    tree = scratch_tree(tmp_path)
    build_py = tree / "oracle" / "build.py"
    text = build_py.read_text()
    flags = '"-O2", "-fopenmp",'
    assert flags in text
    build_py.write_text(text.replace(
        flags, '"-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",'))
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(libasan) and os.path.exists(libasan), "gcc's libasan.so not found"
    env = {"LD_PRELOAD": libasan + (" " + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else ""),
           # python itself is not instrumented: its interned allocations are not leaks of the oracle
           "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
           "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}
    r = run_pins(tree, env, stop_at_first=False)
    out = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, out
    assert "AddressSanitizer" not in out and "runtime error" not in out, out
    # the instrumented library really was the one loaded
    so = tree / "oracle" / "libbnn_oracle.so"
    syms = subprocess.run(["nm", "-D", str(so)], capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms
