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
    ("sign dropped in the decode", "        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */\n    }\n    return sign ? -v : v;",
     "        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */\n    }\n    return v;"),
    ("pairwise split drops an element", "    pairwise(t, x + half, n - half, &s1, &a1);",
     "    pairwise(t, x + half + 1, n - half - 1, &s1, &a1);"),
    ("pairwise split counts an element twice", "    pairwise(t, x + half, n - half, &s1, &a1);",
     "    pairwise(t, x + half - 1, n - half + 1, &s1, &a1);"),
    ("pairwise subtracts the second half", "    pairwise(t, x + half, n - half, &s1, &a1);\n    *s = s0 + s1;",
     "    pairwise(t, x + half, n - half, &s1, &a1);\n    *s = s0 - s1;"),
    ("exact sum: wrong shift", "units = (1024 + f) << (e - 1);", "units = (1024 + f) << e;"),
    ("exact sum: sign ignored", "s += (h & 0x8000) ? -units : units;", "s += units;"),
    ("exact sum: subnormals flushed", "if (e == 0) units = f; ", "if (e == 0) units = 0; "),
    ("int8 read as unsigned", "int64_t v = x[i];", "int64_t v = (uint8_t)x[i];"),
    ("serial loop stops one short", "int redux_oracle_sum_f16_serial(const uint16_t *x, size_t n, double *sum, double *sum_abs)\n{\n    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;\n    const double *t = decode_table();\n    double s = 0.0, a = 0.0;\n    for (size_t i = 0; i < n; ++i) {",
     "int redux_oracle_sum_f16_serial(const uint16_t *x, size_t n, double *sum, double *sum_abs)\n{\n    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;\n    const double *t = decode_table();\n    double s = 0.0, a = 0.0;\n    for (size_t i = 0; i + 1 < n + (n < 3); ++i) {"),
    ("segment results shifted by one element", "redux_oracle_sum_f16(x + s * seglen, seglen, &sum[s], &sum_abs[s]);",
     "redux_oracle_sum_f16(x + s * seglen + (s > 0 && seglen > 0), seglen - (s > 0 && seglen > 0), &sum[s], &sum_abs[s]);"),
    ("pairwise base case skips its first element",
     "if (n <= 128) {\n        double ss = 0.0, aa = 0.0;\n        for (size_t i = 0; i < n; ++i) {\n            double v = t[x[i]];",
     "if (n <= 128) {\n        double ss = 0.0, aa = 0.0;\n        for (size_t i = (n > 100); i < n; ++i) {\n            double v = t[x[i]];"),
    ("sum of |x| forgets the absolute value", "        double v = t[x[i]];\n        s += v;\n        a += fabs(v);\n    }\n    *sum = s;\n    *sum_abs = a;\n    return ORACLE_OK;\n}\n\nstatic void pairwise",
     "        double v = t[x[i]];\n        s += v;\n        a += v;\n    }\n    *sum = s;\n    *sum_abs = a;\n    return ORACLE_OK;\n}\n\nstatic void pairwise"),
    ("chunks of n / T elements: the remainder is lost", "return (size_t)(((unsigned __int128)n * t) / T);", "return (n / T) * t;"),
    ("chunk sums: last chunk left out", "for (int c = 0; c < chunks; ++c) {      /* chunk order, whatever order the threads finished in */",
     "for (int c = 0; c + 1 < chunks + (chunks < 2); ++c) {      /* chunk order, whatever order the threads finished in */"),
    ("int8 chunks start one element late", "(void)redux_oracle_sum_i8(x + lo, hi - lo, &ps[c], &pa[c]);", "(void)redux_oracle_sum_i8(x + lo + (lo > 0), hi - lo - (lo > 0), &ps[c], &pa[c]);"),
]


MUTANTS_MORE = [
    ("bfloat16 exponent bias", "ldexp((double)(128 + f), e - 134)", "ldexp((double)(128 + f), e - 133)"),
    ("bfloat16 subnormal scale", "ldexp((double)f, -133)", "ldexp((double)f, -126)"),
    ("binary32 hidden bit", "ldexp((double)(0x800000u + f), e - 150)", "ldexp((double)(f), e - 150)"),
    ("E4M3 treated as having infinities", "if (e == 15 && f == 7) v = NAN;", "if (e == 15) v = (f == 0) ? INFINITY : NAN;"),
    ("E4M3 bias of E5M2", "ldexp((double)(8 + f), e - 10)", "ldexp((double)(8 + f), e - 18)"),
    ("E5M2 fraction width", "int sign = (b >> 7) & 1, e = (b >> 2) & 0x1f, f = b & 3;\n    double v;", "int sign = (b >> 7) & 1, e = (b >> 2) & 0x1f, f = b & 1;\n    double v;"),
    ("E5M2 subnormal scale", "ldexp((double)f, -16)", "ldexp((double)f, -14)"),
    ("generic pairwise drops an element", "pairwise_any(x, lo + half, n - half, dtype, &s1, &a1);", "pairwise_any(x, lo + half + 1, n - half - 1, dtype, &s1, &a1);"),
    ("generic pairwise ignores its offset", "double v = decode_at(x, lo + i, dtype);", "double v = decode_at(x, i, dtype);"),
    ("8-bit exact sum: wrong shift", "u = e == 0 ? f : (int64_t)(4 + f) << (e - 1);", "u = e == 0 ? f : (int64_t)(4 + f) << e;"),
    ("8-bit exact sum: sign ignored", "s += (b & 0x80) ? -u : u;", "s += u;"),
    ("bfloat16 sign dropped", "else v = ldexp((double)(128 + f), e - 134);              /* (1 + f/128) * 2^(e-127) */\n    return sign ? -v : v;",
     "else v = ldexp((double)(128 + f), e - 134);              /* (1 + f/128) * 2^(e-127) */\n    return v;"),
]


def run_pins(env, test_file, select=None):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", test_file)]
    if select:
        cmd += ["-k", select]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)


@pytest.mark.parametrize("name,old,new", MUTANTS_MORE, ids=[m[0] for m in MUTANTS_MORE])
def test_pins_of_the_other_dtypes_catch_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site not found (or not unique): %r" % old
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", str(lib), str(mutated), "-lm"])
    r = run_pins(dict(os.environ, REDUX_ORACLE_LIB=str(lib)), "test_oracle_pins_more_dtypes.py")
    assert r.returncode == 1, "the pins did not notice: %s\n%s" % (name, r.stdout[-2000:])


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
