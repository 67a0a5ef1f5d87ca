"""The pins must be able to fail: plant one plausible mistake at a time in a
copy of the oracle's C source (CPU only, temporary build) and check that the
pin suite turns red for every one of them."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mhffn_oracle.c")

# (name, text in the source, replacement): dropped terms, wrong signs, wrong indices,
# transposed operands, accumulators that do not restart
MUTATIONS = [
    ("eps_dropped", "r[e] = s[e] / (Z + eps);", "r[e] = s[e] / Z;"),
    ("softmax_instead_of_sigmoid", "s[e] = sigmoid_f64(p[e]);", "s[e] = exp(p[e]);"),
    ("gate_logit_transposed", "p[e] += qj * w[e];", "p[e] += qj * Wr_h[(size_t)e * d_h + j < (size_t)d_h * E ? (size_t)e * d_h + j : 0];"),
    ("silu_without_gate_factor", "const double a = g * sigmoid_f64(g) * u;\n            const double* v = V", "const double a = sigmoid_f64(g) * u;\n            const double* v = V"),
    ("up_and_gate_swapped", "const double g = dot_f64(q, K + (size_t)c * dh, dh);\n            const double u = dot_f64(q, U + (size_t)c * dh, dh);\n            const double a = g * sigmoid_f64(g) * u;\n            const double* v = V",
     "const double u = dot_f64(q, K + (size_t)c * dh, dh);\n            const double g = dot_f64(q, U + (size_t)c * dh, dh);\n            const double a = g * sigmoid_f64(g) * u;\n            const double* v = V"),
    ("weights_not_applied", "for (int j = 0; j < dh; ++j) y[j] += r[e] * ye[j];", "for (int j = 0; j < dh; ++j) y[j] += ye[j];"),
    ("head_offset_wrong", "const double* q = X + l * ldx + (size_t)h * dh; /* split_H */", "const double* q = X + l * ldx + (size_t)((h + 1) % H) * dh; /* split_H */"),
    ("dr_not_restarted", "double dre = 0.0;\n          for (int c = 0; c < de; ++c) {", "static __thread double dre_keep = 0.0; double dre = (e == 0) ? 0.0 : dre_keep;\n          for (int c = 0; c < de; ++c) {"),
    ("silu_derivative_term_dropped", "const double dm = r[e] * da * u * (sg + g * sg * (1.0 - sg));\n#pragma omp simd\n            for (int j = 0; j < dh; ++j) dq[j]", "const double dm = r[e] * da * u * sg;\n#pragma omp simd\n            for (int j = 0; j < dh; ++j) dq[j]"),
    ("routing_grad_sign", "const double ds = (dr[e] - dot_dr_r) / (Z + d->eps);", "const double ds = (dr[e] + dot_dr_r) / (Z + d->eps);"),
    ("routing_term_of_dx_dropped", "dq[j] += acc;", "dq[j] += 0.0 * acc;"),
    ("dv_uses_ungated_activation", "const double ra = re * a; /* gated activation */", "const double ra = a; /* gated activation */"),
    ("dk_du_swapped", "dk[j] += dm * q[j];   /* dK += dM^T Q       */\n                  du[j] += dn * q[j];", "dk[j] += dn * q[j];   /* dK += dM^T Q       */\n                  du[j] += dm * q[j];"),
    ("dwr_missing_sigmoid_derivative", "dp[e] = ds * s[e] * (1.0 - s[e]);", "dp[e] = ds;"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(name, old, new):
    src = open(SRC).read()
    if name == "dr_not_restarted":
        new = new.replace("(e == 0) ? 0.0 : dre_keep", "(e == 0) ? 0.0 : dre_keep")
    assert src.count(old) >= 1, "mutation target not found: %s" % name
    mutated = src.replace(old, new, 1)
    if name == "dr_not_restarted":
        mutated = mutated.replace("dr[e] = dre;", "dr[e] = dre; dre_keep = dre;", 1)
    with tempfile.TemporaryDirectory() as tmp:
        c = os.path.join(tmp, "mut.c")
        lib = os.path.join(tmp, "libmut.so")
        open(c, "w").write(mutated)
        subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=gnu11",
                               "-I", os.path.join(ROOT, "oracle"), "-o", lib, c, "-lm"])
        env = dict(os.environ, MHFFN_ORACLE_LIB=lib, MHFFN_ORACLE_MUTATION_HARNESS="tests/test_oracle_pins.py", OMP_NUM_THREADS="2")
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                           cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert "failed" in r.stdout, r.stdout[-500:]


def test_unmutated_oracle_passes_the_same_harness():
    """Guards the harness itself: the same subprocess call is green without a mutation."""
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "libclean.so")
        subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=gnu11",
                               "-I", os.path.join(ROOT, "oracle"), "-o", lib, SRC, "-lm"])
        env = dict(os.environ, MHFFN_ORACLE_LIB=lib, MHFFN_ORACLE_MUTATION_HARNESS="tests/test_oracle_pins.py", OMP_NUM_THREADS="2")
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                           cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-800:]


# ---- the module oracle (Python around the C oracle): same idea, on a copy of the package ----
MODULE_SRC = os.path.join(ROOT, "oracle", "mhffn_oracle.py")
MODULE_MUTATIONS = [
    ("w_in_transposed", "Q = X @ W_in\n", "Q = X @ W_in.T\n"),
    ("w_out_transposed", "O = S @ W_out\n", "O = S @ W_out.T\n"),
    ("ds_without_transpose", "dS = dO @ W_out.T", "dS = dO @ W_out"),
    ("dw_in_from_projected_input", '"dW_in": X.T @ g["dX"]', '"dW_in": Q.T @ g["dX"]'),
    ("dw_out_from_path_input", '"dW_out": S.T @ dO', '"dW_out": Q.T @ dO'),
    ("dx_without_input_projection", '"dX": g["dX"] @ W_in.T', '"dX": g["dX"]'),
]


def _run_module_pins(tmp, py_source):
    import shutil
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tmp, "oracle"),
                    ignore=shutil.ignore_patterns("__pycache__"))
    open(os.path.join(tmp, "oracle", "mhffn_oracle.py"), "w").write(py_source)
    os.makedirs(os.path.join(tmp, "tests"))
    for f in ("__init__.py", "conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(tmp, "tests", f))
    env = dict(os.environ, OMP_NUM_THREADS="2", PYTHONPATH=tmp)
    env.pop("MHFFN_ORACLE_LIB", None)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           "-k", "module", os.path.join(tmp, "tests", "test_oracle_pins.py")],
                          cwd=tmp, env=env, capture_output=True, text=True)


@pytest.mark.parametrize("name,old,new", MODULE_MUTATIONS, ids=[m[0] for m in MODULE_MUTATIONS])
def test_module_pins_catch_planted_mistake(name, old, new):
    src = open(MODULE_SRC).read()
    assert src.count(old) >= 1, "mutation target not found: %s" % name
    with tempfile.TemporaryDirectory() as tmp:
        r = _run_module_pins(tmp, src.replace(old, new))
    assert r.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert "failed" in r.stdout, r.stdout[-500:]


def test_unmutated_module_oracle_passes_the_same_harness():
    with tempfile.TemporaryDirectory() as tmp:
        r = _run_module_pins(tmp, open(MODULE_SRC).read())
    assert r.returncode == 0 and "passed" in r.stdout, r.stdout[-800:]
