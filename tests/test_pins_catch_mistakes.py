"""The pins must be able to fail: each plausible mistake planted in a copy of the oracle's C
source (a wrong sign, a dropped scale, a wrong head map, an off-by-one mask, a transposed
operand ...) has to make the pin suite fail.  Runs entirely on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "matkv_oracle.c")

MUTANTS = {
    "rope-sign": ("x[j] = a * c - b * s;", "x[j] = a * c + b * s;"),
    "rope-pairing-adjacent": ("double a = x[j], b = x[j + half];", "double a = x[j], b = x[(j + 1) % D];"),
    "rope-frequency": ("pow(base, -2.0 * (double)j / (double)D)", "pow(base, -1.0 * (double)j / (double)D)"),
    "rope-position-offset": ("oracle_rope(k, D, pos0 + (double)i, base);", "oracle_rope(k, D, pos0 + (double)i + 1.0, base);"),
    "v-rotated-too": ("oracle_rope(k, D, pos0 + (double)i, base);",
                      "oracle_rope(k, D, pos0 + (double)i, base); oracle_rope(v, D, pos0 + (double)i, base);"),
    "projection-transposed": ("const double* wk = Wk + ((size_t)g * D + d) * Hd;", "const double* wk = Wk + ((size_t)d * Hkv + g) * Hd;"),
    "scale-dropped": ("s[n] = acc * scale;", "s[n] = acc;"),
    "gqa-interleaved": ("int g = h / G;", "int g = h % Hkv;"),
    "mask-off-by-one": ("int visible = n_ctx + row0 + r + 1;", "int visible = n_ctx + row0 + r;"),
    "mask-ignores-row": ("int visible = n_ctx + row0 + r + 1;", "int visible = n_ctx + row0 + R;"),
    "softmax-no-normalisation": ("double p = s[n] / den;", "double p = s[n];"),
    "value-of-wrong-head": ("const double* v = V + ((size_t)g * Nk + n) * D;", "const double* v = V + ((size_t)0 * Nk + n) * D;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    c = tmp_path / "mutant.c"
    c.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(c), "-lm"], check=True)
    env = dict(os.environ, MATKV_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0, f"the pins did not notice the planted mistake '{name}'"


def test_unmutated_oracle_passes_the_same_way(tmp_path):
    lib = tmp_path / "libclean.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), SRC, "-lm"], check=True)
    env = dict(os.environ, MATKV_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-2000:]


# Mistakes planted in the Python part of the oracle (the compressed-blob arithmetic and the
# glue around the C routines): the pins run in a copy of the tree that holds the mutated module.
PY_SRC = os.path.join(ROOT, "oracle", "matkv_oracle.py")

PY_MUTANTS = {
    "e4m3-truncates": ("q = np.rint((an / np.exp2(e) - 1.0) * 8.0)", "q = np.floor((an / np.exp2(e) - 1.0) * 8.0)"),
    "e4m3-bias-8": ("code = np.where(sub, q_sub, (e + 7) * 8 + q).astype(np.int64)", "code = np.where(sub, q_sub, (e + 8) * 8 + q).astype(np.int64)"),
    "e4m3-no-subnormals": ("sub = a < 2.0 ** -6", "sub = a < 0.0"),
    "e4m3-saturates-one-code-late": ("code = np.minimum(code, 0x7E)", "code = np.minimum(np.where(np.abs(y) > 448.0, 0x7F, code), 0x7F)"),
    "e4m3-decode-mantissa-4-bits": ("(1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))", "(1.0 + m / 16.0) * np.exp2((e - 7).astype(np.float64))"),
    "e4m3-decode-has-infinity": ("val = np.where((e == 15) & (m == 7), np.nan, val)", "val = np.where(e == 15, np.nan, val)"),
    "scale-boundary-at-2": ("k = np.maximum(np.where(2.0 * m <= 1.75, e - 1 - 8, e - 1 - 7), -60)", "k = np.maximum(np.where(2.0 * m <= 2.0, e - 1 - 8, e - 1 - 7), -60)"),
    "scale-targets-240": ("k = np.maximum(np.where(2.0 * m <= 1.75, e - 1 - 8, e - 1 - 7), -60)", "k = np.maximum(np.where(2.0 * m <= 1.875, e - 1 - 7, e - 1 - 6), -60)"),
    "scale-per-tensor": ("scales = kv_scale(np.abs(X).max(axis=(2, 3)))", "scales = kv_scale(np.abs(X).max(axis=(1, 2, 3), keepdims=True) * np.ones((2, X.shape[1])))"),
    "decompress-forgets-scale": ("X = e4m3_decode(codes) * _f64(scales)[:, :, None, None]", "X = e4m3_decode(codes)"),
    "chunk-attn-not-causal": ("return attn(Q, K, V, 0, 0, scale)", "return attn(Q, K, V, np.asarray(K).shape[1], 0, scale)"),
    "store-round-truncates": ("bias = np.uint64((1 << 44) - 1) + ((u >> np.uint64(45)) & np.uint64(1))", "bias = np.uint64(0)"),
    "assemble-tail-first": ("ks = [_f64(k) for k, _ in chunks] + [_f64(tail_k)]", "ks = [_f64(tail_k)] + [_f64(k) for k, _ in chunks]"),
}


def _run_pins_in_copy(tmp_path, py_source):
    import shutil
    tree = tmp_path / "tree"
    shutil.copytree(os.path.join(ROOT, "oracle"), tree / "oracle", ignore=shutil.ignore_patterns("__pycache__"))
    (tree / "oracle" / "matkv_oracle.py").write_text(py_source)
    (tree / "tests").mkdir()
    for name in ("conftest.py", "test_oracle_pins.py", "__init__.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), tree / "tests" / name)
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), tree / "tests" / "golden")
    env = {k: v for k, v in os.environ.items() if k != "MATKV_ORACLE_LIB"}
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pins.py"],
                          cwd=str(tree), env=env, capture_output=True, text=True)


@pytest.mark.parametrize("name", sorted(PY_MUTANTS))
def test_planted_python_mistake_is_caught(name, tmp_path):
    old, new = PY_MUTANTS[name]
    src = open(PY_SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    r = _run_pins_in_copy(tmp_path, src.replace(old, new))
    assert r.returncode != 0, f"the pins did not notice the planted mistake '{name}'"
    assert "passed" not in r.stdout.splitlines()[-1] or "failed" in r.stdout, r.stdout[-500:]


def test_unmutated_python_oracle_passes_in_a_copy(tmp_path):
    r = _run_pins_in_copy(tmp_path, open(PY_SRC).read())
    assert r.returncode == 0, r.stdout[-2000:]
