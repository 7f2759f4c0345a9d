"""The pins must catch plausible mistakes: each mutant below is a copy of redux_oracle.c with one
planted bug (on the CPU, in the oracle only); the pin suite has to fail on every one of them."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "redux_oracle.c")

MUTANTS = [
    ("wrong exponent bias", "ldexp((double)(1024 + f), e - 25)", "ldexp((double)(1024 + f), e - 24)"),
    ("wrong subnormal scale", "ldexp((double)f, -24)", "ldexp((double)f, -23)"),
    ("hidden bit off by one", "ldexp((double)(1024 + f), e - 25)", "ldexp((double)(1023 + f), e - 25)"),
    ("sign dropped in the decode", "return sign ? -v : v;", "return v;"),
    ("pairwise split drops an element", "pairwise(t, x + half, n - half, &s1, &a1);",
     "pairwise(t, x + half + 1, n - half - 1, &s1, &a1);"),
    ("pairwise split counts an element twice", "pairwise(t, x + half, n - half, &s1, &a1);",
     "pairwise(t, x + half - 1, n - half + 1, &s1, &a1);"),
    ("pairwise base case skips its first element",
     "if (n <= 128) {\n        double ss = 0.0, aa = 0.0;\n        for (size_t i = 0; i < n; ++i) {",
     "if (n <= 128) {\n        double ss = 0.0, aa = 0.0;\n        for (size_t i = (n > 100); i < n; ++i) {"),
    ("pairwise subtracts the second half", "*s = s0 + s1;", "*s = s0 - s1;"),
    ("exact sum: wrong shift", "units = (1024 + f) << (e - 1);", "units = (1024 + f) << e;"),
    ("exact sum: sign ignored", "s += (h & 0x8000) ? -units : units;", "s += units;"),
    ("exact sum: subnormals flushed", "if (e == 0) units = f; ", "if (e == 0) units = 0; "),
    ("int8 read as unsigned", "int64_t v = x[i];", "int64_t v = (uint8_t)x[i];"),
    ("serial loop stops one short", "int redux_oracle_sum_f16_serial(const uint16_t *x, size_t n, double *sum, double *sum_abs)\n{\n    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;\n    const double *t = decode_table();\n    double s = 0.0, a = 0.0;\n    for (size_t i = 0; i < n; ++i) {",
     "int redux_oracle_sum_f16_serial(const uint16_t *x, size_t n, double *sum, double *sum_abs)\n{\n    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;\n    const double *t = decode_table();\n    double s = 0.0, a = 0.0;\n    for (size_t i = 0; i + 1 < n + (n < 3); ++i) {"),
    ("segment results shifted by one element", "redux_oracle_sum_f16(x + s * seglen, seglen, &sum[s], &sum_abs[s]);",
     "redux_oracle_sum_f16(x + s * seglen + (s > 0 && seglen > 0), seglen - (s > 0 && seglen > 0), &sum[s], &sum_abs[s]);"),
    ("sum of |x| forgets the absolute value", "        double v = t[x[i]];\n        s += v;\n        a += fabs(v);\n    }\n    *sum = s;\n    *sum_abs = a;\n    return ORACLE_OK;\n}\n\nstatic void pairwise",
     "        double v = t[x[i]];\n        s += v;\n        a += v;\n    }\n    *sum = s;\n    *sum_abs = a;\n    return ORACLE_OK;\n}\n\nstatic void pairwise"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site not found (or not unique): %r" % old
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", str(lib), str(mutated), "-lm"])
    env = dict(os.environ, REDUX_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k", "not large"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 1, "the pins did not notice: %s\n%s" % (name, r.stdout[-2000:])


def test_unmutated_oracle_passes_the_same_selection():
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k", "not large"],
                       cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
