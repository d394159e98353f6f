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
