"""Do the pins have teeth?  Plant one plausible mistake at a time in a copy of the oracle's
source (on the CPU, never in the HIP path) and check that the pin tests then fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ftk_oracle.cpp")

MUTANTS = [
    ("loo-includes-own-mode", "if (k != n) prod *= t.c[k][r];", "prod *= t.c[k][r];"),
    ("a-gradient-sign", "drow[j] += -e * t.gs[n][j]", "drow[j] += e * t.gs[n][j]"),
    ("a-regulariser-dropped", "+ (double)lambda_A * (double)a[n][j];", ";"),
    ("b-gradient-not-averaged", "GB[n][q] / (double)n_samples", "GB[n][q]"),
    ("b-regulariser-dropped", "+ (double)lambda_B * (double)B[n][q]));", "));"),
    ("b-transposed-in-c", "acc += (double)a[n][j] * (double)B[n][(size_t)j * R + r];",
     "acc += (double)a[n][j] * (double)B[n][((size_t)r * J[n] + j) % ((size_t)J[n] * R)];"),
    ("b-gradient-uses-c-not-w", "-e * (double)a[n][j] * t.w[n][r];", "-e * (double)a[n][j] * t.c[n][r];"),
    ("error-sign", "const double e = (double)vals[p] - t.xhat;\n        for (int n = 0; n < N; ++n) {\n            const size_t i",
     "const double e = t.xhat - (double)vals[p];\n        for (int n = 0; n < N; ++n) {\n            const size_t i"),
    ("philox-words-swapped", "(k & 1u) ? ((uint64_t)o.w[2] | ((uint64_t)o.w[3] << 32))", "(k & 1u) ? ((uint64_t)o.w[3] | ((uint64_t)o.w[2] << 32))"),
    ("position-by-modulo", "return mulhi_u64(u, nnz);", "return u % nnz;"),
    ("philox-nine-rounds", "round < 10", "round < 9"),
    ("init-uses-low-bits", "(o.w[0] >> 8)", "(o.w[0] & 0xFFFFFFu)"),
    ("untouched-rows-decay", "if (!touched[n][(size_t)i]) continue;",
     "if (!touched[n][(size_t)i]) { for (int j = 0; j < J[n]; ++j) A[n][(size_t)i * J[n] + j] *= (float)(1.0 - lr_A * lambda_A); continue; }"),
    ("in-place-step-uses-stale-rows", "            nonzero_terms(N, J, R, a.data(), B, t);   // everything from the current rows\n",
     "            if (n == 0) nonzero_terms(N, J, R, a.data(), B, t);\n"),
    ("in-place-core-not-averaged", "(double)lr_B * (GB[n][q] / (double)n_samples + (double)lambda_B * (double)B[n][q]));\n    return 0;\n}\n\n// Summed",
     "(double)lr_B * (GB[n][q] + (double)lambda_B * (double)B[n][q]));\n    return 0;\n}\n\n// Summed"),
    ("rmse-without-root", "*rmse_out = std::sqrt(sse / (double)m);", "*rmse_out = sse / (double)m;"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    # the synchronous step comes first in the file; a snippet it shares with the in-place step is
    # mutated there only (the in-place step has mutants of its own)
    assert text.count(old) in (1, 2), "mutation site for %s not found" % name
    mutant = tmp_path / "mutant.cpp"
    mutant.write_text(text.replace(old, new, 1))
    env = dict(os.environ, FTK_ORACLE_SOURCE=str(mutant), FTK_ORACLE_LIB=str(tmp_path / "libmutant.so"))
    proc = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", "test_oracle_sampling.py"),
                           os.path.join(ROOT, "tests", "test_oracle_model.py")],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 1, "pins did not catch mutant %s:\n%s" % (name, proc.stdout[-2000:])
    assert "failed" in proc.stdout
