"""The pins must reject plausible mistakes in the oracle.

Each case below plants one mistake in a copy of oracle/corr_oracle.c (a swapped
index, a dropped term, a wrong border rule ...), builds it, and runs the pin
tests against that build in a child process: at least one pin has to fail.
The mistakes live only in temporary copies on the CPU.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "corr_oracle.c")

# (name, text in the oracle source, what it becomes)
MUTANTS = [
    ("x and y offsets of a tap swapped",
     "const double sx = cx * inv + (double)(i - r);\n    const double sy = cy * inv + (double)(j - r);",
     "const double sx = cx * inv + (double)(j - r);\n    const double sy = cy * inv + (double)(i - r);"),
    ("x and y coordinate channels swapped",
     "const double cx = (double)coords[(((size_t)b * 2 + 0) * H + y) * W + x];\n"
     "    const double cy = (double)coords[(((size_t)b * 2 + 1) * H + y) * W + x];",
     "const double cx = (double)coords[(((size_t)b * 2 + 1) * H + y) * W + x];\n"
     "    const double cy = (double)coords[(((size_t)b * 2 + 0) * H + y) * W + x];"),
    ("two corners of the bilinear stencil swapped",
     "wx * (1.0 - wy) * c01\n         + (1.0 - wx) * wy * c10",
     "wx * (1.0 - wy) * c10\n         + (1.0 - wx) * wy * c01"),
    ("coordinates not scaled per level", "const double inv = ldexp(1.0, -l);", "const double inv = 1.0;"),
    ("level scale 2^-(l+1)", "const double inv = ldexp(1.0, -l);", "const double inv = ldexp(1.0, -l - 1);"),
    ("pooling takes one element twice", "src[r1] + src[r1 + D]);", "src[r1] + src[r1]);"),
    ("pooling averages with 1/2", "0.25 * (src[r0]", "0.5 * (src[r0]"),
    ("1/sqrt(D) dropped", "return s * scale;", "return s;"),
    ("border clamped instead of zero padded",
     "if (v < 0 || u < 0 || v >= p->H[l] || u >= p->W[l]) return 0.0;",
     "if (v < 0) v = 0; if (u < 0) u = 0; if (v >= p->H[l]) v = p->H[l] - 1; if (u >= p->W[l]) u = p->W[l] - 1;"),
    ("truncation instead of floor", "const double fx0 = floor(sx), fy0 = floor(sy);",
     "const double fx0 = trunc(sx), fy0 = trunc(sy);"),
    ("window starts one pixel late", "(double)(i - r);", "(double)(i - r + 1);"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_a_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "the oracle source no longer contains the text this case edits"
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                           "-o", str(lib), str(mutant_c), "-lm"])
    env = dict(os.environ, CORR_ORACLE_LIB_OVERRIDE=str(lib), OMP_NUM_THREADS="4")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 1, "no pin failed for: %s\n%s" % (name, run.stdout[-2000:])
    assert "failed" in run.stdout


def test_the_unmodified_oracle_passes_through_the_same_route(tmp_path):
    lib = tmp_path / "libclean.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                           "-o", str(lib), SRC, "-lm"])
    env = dict(os.environ, CORR_ORACLE_LIB_OVERRIDE=str(lib), OMP_NUM_THREADS="4")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:]


# ---- the gradient oracle (oracle/corr_oracle_backward.c), against tests/test_oracle_backward_pins.py
SRC_BACKWARD = os.path.join(ROOT, "oracle", "corr_oracle_backward.c")
BACKWARD_MUTANTS = [
    ("corner weights of x and y swapped", "const double w = (cxi ? wx : 1.0 - wx) * (cyi ? wy : 1.0 - wy);",
     "const double w = (cxi ? wy : 1.0 - wy) * (cyi ? wx : 1.0 - wx);"),
    ("pooling adjoint spreads with 1/2", "const double t = 0.25 * dlev[l]", "const double t = 0.5 * dlev[l]"),
    ("pooling adjoint reaches one pixel only", "for (int a2 = 0; a2 < 2; ++a2)", "for (int a2 = 0; a2 < 1; ++a2)"),
    ("1/sqrt(D) dropped", "const double gw = g * w * scale;", "const double gw = g * w;"),
    ("gradient of fmap1 misses the level's features", "+= gw * lev[l][q + d];", "+= gw * lev[0][q + d];"),
    ("corners on the last column skipped",
     "if (u < 0 || v < 0 || u >= Wl[l] || v >= Hl[l]) continue;     /* zero padding: no dependence */",
     "if (u < 0 || v < 0 || u >= Wl[l] - 1 || v >= Hl[l]) continue;"),
    ("tap offsets swapped", "const double sx = cx * ldexp(1.0, -l) + (double)(i - r);\n"
     "                            const double sy = cy * ldexp(1.0, -l) + (double)(j - r);",
     "const double sx = cx * ldexp(1.0, -l) + (double)(j - r);\n"
     "                            const double sy = cy * ldexp(1.0, -l) + (double)(i - r);"),
]

@pytest.mark.parametrize("name,old,new", BACKWARD_MUTANTS, ids=[m[0] for m in BACKWARD_MUTANTS])
def test_backward_pins_reject_a_planted_mistake(tmp_path, name, old, new):
    src = open(SRC_BACKWARD).read()
    assert src.count(old) == 1, "the oracle source no longer contains the text this case edits"
    mutant_c = tmp_path / "mutant_backward.c"
    mutant_c.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                           "-o", str(lib), SRC, str(mutant_c), "-lm"])
    env = dict(os.environ, CORR_ORACLE_LIB_OVERRIDE=str(lib), OMP_NUM_THREADS="4")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_backward_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 1, "no pin failed for: %s\n%s" % (name, run.stdout[-2000:])
    assert "failed" in run.stdout
