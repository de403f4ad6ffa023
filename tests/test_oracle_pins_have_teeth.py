"""Mutation check of the oracle's pins, on the CPU: one plausible mistake at a time is planted in
a COPY of the C oracle (dropped normalisation, wrong head map, wrong sign, off-by-one mask, K read
for V, ...), the copy is compiled, and the pin tests are run against it in a subprocess.  Every
mutant must be rejected by at least one pin; the unmodified copy must pass."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "orbit_oracle.c")

PV_LOOP = ("for (int64_t t = 0; t < n; ++t) {\n"
           "    const uint16_t *base = arena + (int64_t)pages[t / P] * page_elems;")
PAGE_LOOKUP = ("int32_t pg = pages[t / P];\n"
               "    if (pg < 0 || pg >= arena_pages) { if (!weights) free(s); return -3; }")

MUTANTS = [
    ("control", None, None),
    ("head map by modulo instead of contiguous groups", "const int g = h / (Hq / Hkv);", "const int g = h % Hkv;"),
    ("default scale 1/D", "scale = 1.0 / sqrt((double)D);", "scale = 1.0 / (double)D;"),
    ("no max subtraction", "s[t] = exp(s[t] - mx);", "s[t] = exp(s[t]);"),
    ("no normalisation", "s[t] /= z;", "s[t] /= 1.0;"),
    ("last token dropped from P.V", PV_LOOP, PV_LOOP.replace("t < n;", "t + 1 < n || t == 0;")),
    ("V read through the K offset", "base[v_offset(g, (int)(t % P), d, P, D, Hkv)]);\n  }\n  if (!weights)",
     "base[k_offset(g, (int)(t % P), d, P, D)]);\n  }\n  if (!weights)"),
    ("score of token t taken from the page of token t+1", PAGE_LOOKUP,
     PAGE_LOOKUP.replace("pages[t / P]", "pages[(t + 1) / P < (n + P - 1) / P ? (t + 1) / P : t / P]")),
    ("dot product over D-1 dims", "for (int d = 0; d < D; ++d)\n      dot +=", "for (int d = 0; d + 1 < D; ++d)\n      dot +="),
    ("sign of the score", "s[t] = scale * dot;", "s[t] = -scale * dot;"),
]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_a_planted_mistake(tmp_path, name, old, new):
    with open(SRC) as f:
        src = f.read()
    if old is not None:
        assert src.count(old) >= 1, "mutation site not found: " + name
        src = src.replace(old, new)
    c = tmp_path / "mutant.c"
    c.write_text(src)
    lib = str(tmp_path / "libmutant.so")
    subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", lib, str(c), "-lm"], check=True)
    env = dict(os.environ, ORBIT_ORACLE_LIB=lib)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    if old is None:
        assert res.returncode == 0, res.stdout[-2000:]
    else:
        assert res.returncode == 1 and "FAILED" in res.stdout, f"pins accepted the mutant '{name}':\n" + res.stdout[-1500:]
