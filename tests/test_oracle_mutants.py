"""The pins must bite: each plausible slip, planted in a copy of the oracle source (never in the
oracle itself, and only on the CPU), has to make the pin suite fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "obrs_oracle.c")

MUTANTS = [
    ("acceptance uses q/p instead of p/q",
     "double r = exp(out->logratio) / lambda;", "double r = exp(-out->logratio) / lambda;"),
    ("acceptance forgets lambda",
     "double r = exp(out->logratio) / lambda;", "double r = exp(out->logratio);"),
    ("mask uses <= instead of <",
     "out->mask = (u < out->accept) ? 1 : 0;", "out->mask = (u <= out->accept) ? 1 : 0;"),
    ("kept mass divides q by lambda instead of p",
     "double qv = exp(logq_v);\n    double pv = exp(logp_v) / lambda;",
     "double qv = exp(logq_v) / lambda;\n    double pv = exp(logp_v);"),
    ("kept mass takes the max",
     "return qv < pv ? qv : pv;", "return qv > pv ? qv : pv;"),
    ("ties go to the highest id",
     "return (ia > ib) - (ia < ib);", "return (ia < ib) - (ia > ib);"),
    ("top-k sorts ascending",
     "if (va > vb) return -1;\n    if (va < vb) return 1;", "if (va > vb) return 1;\n    if (va < vb) return -1;"),
    ("union counts a shared token twice",
     "if (in_union[v]) {\n            z_approx += t;", "if (in_union[v]) {\n            z_approx += t * (double)in_union[v];"),
    ("union forgets the policy list",
     "for (int32_t j = 0; j < k; ++j) in_union[kp[j]] = 1;", ""),
    ("log-sum-exp drops the max shift",
     "return m + log(s);", "return log(s);"),
    ("log-ratio has the wrong sign",
     "out->logratio = out->logp_x - out->logq_x;", "out->logratio = out->logq_x - out->logp_x;"),
    ("alpha_hat divides by all rows, padding included",
     "b->alpha_hat = (double)b->n_accept / n;", "b->alpha_hat = (double)b->n_accept / (double)T;"),
    ("kappa is inverted",
     "b->kappa = alpha / b->mean_z_approx;", "b->kappa = b->mean_z_approx / alpha;"),
    ("weight uses min(lambda, ratio)",
     "double w = z_t * (lambda > ratio ? lambda : ratio);", "double w = z_t * (lambda < ratio ? lambda : ratio);"),
    ("rho clips the reference factor from below",
     "rho *= rr < c2 ? rr : c2;", "rho *= rr > c2 ? rr : c2;"),
    ("KL(p||q) weights by q",
     "kl_pq += pv * (logp_v - logq_v);", "kl_pq += exp(logq_v) * (logp_v - logq_v);"),
    ("stored form: the k-th bound takes the largest stored value",
     "if (n == 0 || logq_ids[j] < kth) kth = logq_ids[j];", "if (n == 0 || logq_ids[j] > kth) kth = logq_ids[j];"),
    ("stored form: a repeated id is counted twice",
     "if (v < 0 || v >= V || stored[v]) continue;", "if (v < 0 || v >= V) continue;"),
    ("stored form: the even share ignores the stored mass",
     "double rest = 1.0 - mass;", "double rest = 1.0;"),
    ("stored form: tokens of TopK_new outside the stored list are dropped under every rule",
     "z += kept_mass(tail, lp[v] - lse_p, lambda);\n            ++usize;", "++usize;"),
    ("band adjustment keeps the weights outside the band",
     "return (w >= lo && w <= hi) ? w : 0.0;", "return (w >= lo && w <= hi) ? 0.0 : w;"),
    ("identity adjustment still truncates",
     "if (f_mode == JPO_F_IDENTITY) return w;", "if (f_mode == JPO_F_IDENTITY) return w < c1 ? w : c1;"),
    ("token log-probability forgets the log-sum-exp",
     "out[t] = l[x[t]] - jpo_logsumexp(l, V);", "out[t] = l[x[t]];"),
    ("budget solver: solves A + B lambda = abar instead of A + B / lambda",
     "lambda = B / (abar - A);", "lambda = (abar - A) / B;"),
    ("budget solver: keeps the mass of q at or below the piece in A",
     "A -= e[i].q;\n        B += e[i].p;", "B += e[i].p;"),
    ("budget solver: budget 1 returns the largest ratio",
     "if (abar >= A) { lambda = e[0].r; return lambda; }", "if (abar >= A) { lambda = e[n - 1].r; return lambda; }"),
    ("batch budget solver: rows are not weighted by 1/n",
     "e[n].q = q / (double)n_rows;\n            e[n].p = p / (double)n_rows;", "e[n].q = q;\n            e[n].p = p;"),
    ("batch budget solver: the mean runs over padding rows too",
     "for (int64_t t = 0; t < T; ++t) n_rows += x[t] >= 0 ? 1 : 0;", "for (int64_t t = 0; t < T; ++t) n_rows += 1;"),
    ("distillation gradient has the wrong sign",
     "out[v] = weight * (exp(lq[v] - lse_q) - exp(lp[v] - lse_p));", "out[v] = weight * (exp(lp[v] - lse_p) - exp(lq[v] - lse_q));"),
    ("distillation gradient drops the row weight",
     "jpo_distill_grad_row(lq, lp, V, scale * (row_scale ? (double)row_scale[t] : 1.0), o);", "jpo_distill_grad_row(lq, lp, V, scale, o);"),
    ("a sampled id outside the vocabulary is taken as a padding row with zero results",
     "out->z_approx = out->z_exact = out->kl_p_q = out->kl_p_qtilde = NAN;\n        return;\n    }\n    out->valid = 1;\n\n",
     "return;\n    }\n    out->valid = 1;\n\n"),
    ("distillation gradient fills padding rows",
     "if (x[t] < 0 || x[t] >= V || !isfinite(lse_q) || !isfinite(lse_p)) {", "if (x[t] >= V || !isfinite(lse_q) || !isfinite(lse_p)) {"),
]


def test_mutant_snippets_exist_in_the_oracle():
    src = open(SRC).read()
    for name, old, _ in MUTANTS:
        assert src.count(old) == 1, name
    # the in_union marks are 0/1, so the "counted twice" mutant needs them to accumulate
    assert "in_union[kq[j]] = 1;" in src


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    if name == "union counts a shared token twice":
        src = src.replace("in_union[kq[j]] = 1;", "in_union[kq[j]] += 1;").replace("in_union[kp[j]] = 1;", "in_union[kp[j]] += 1;")
    src = src.replace(old, new)
    c = tmp_path / "mutant.c"
    so = tmp_path / "libmutant.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", str(c), "-o", str(so), "-lm"], check=True)
    env = dict(os.environ, JPO_ORACLE_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"no pin caught: {name}"
    assert "failed" in r.stdout, r.stdout[-500:]


# ---- the Python part of the oracle (the fused lm_head form's logits) -------------------------------
PY_SRC = os.path.join(ROOT, "oracle", "obrs_oracle.py")

PY_MUTANTS = [
    ("lm_head logits: bf16 bits widened by the wrong shift",
     "(a.astype(np.uint32) << 16)", "(a.astype(np.uint32) << 15)"),
    ("lm_head logits: bf16 bits taken as integers",
     "return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)", "return a.astype(np.float64)"),
    ("lm_head logits: the projection is used transposed",
     "return wide(H) @ wide(W)", "return wide(H) @ wide(W).T"),
    ("lm_head logits: the product is taken in float32",
     "return wide(H) @ wide(W)", "return (wide(H).astype(np.float32) @ wide(W).astype(np.float32)).astype(np.float64)"),
]

_RUNNER = """
import importlib.util, sys
sys.path.insert(0, {root!r})
import oracle
spec = importlib.util.spec_from_file_location("oracle.obrs_oracle", {mutant!r})
m = importlib.util.module_from_spec(spec)
sys.modules["oracle.obrs_oracle"] = m
spec.loader.exec_module(m)
oracle.obrs_oracle = m
import pytest
sys.exit(pytest.main([{pins!r}, "-x", "-q", "-p", "no:cacheprovider", "-k", "lm_head"]))
"""


def test_python_mutant_snippets_exist_in_the_oracle():
    src = open(PY_SRC).read()
    for name, old, _ in PY_MUTANTS:
        assert src.count(old) == 1, name


@pytest.mark.parametrize("name,old,new", PY_MUTANTS,
                         ids=[m[0] for m in PY_MUTANTS])
def test_pins_catch_planted_mistake_in_the_python_part(tmp_path, name, old, new):
    from oracle import obrs_oracle as real
    mutant = tmp_path / "obrs_oracle_mutant.py"
    mutant.write_text(open(PY_SRC).read().replace(old, new))
    # the mutant module sits outside the oracle folder: point it at the built C library
    env = dict(os.environ, JPO_ORACLE_LIB=real.build())
    pins = os.path.join(ROOT, "tests", "test_oracle_pins.py")
    r = subprocess.run([sys.executable, "-c", _RUNNER.format(root=ROOT, mutant=str(mutant), pins=pins)],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"no pin caught: {name}"
    assert "failed" in r.stdout, r.stdout[-500:]


def test_unmutated_python_part_passes_through_the_same_runner(tmp_path):
    """The runner itself must not be what fails: the unchanged source passes the same pins."""
    from oracle import obrs_oracle as real
    copy = tmp_path / "obrs_oracle_copy.py"
    copy.write_text(open(PY_SRC).read())
    env = dict(os.environ, JPO_ORACLE_LIB=real.build())
    pins = os.path.join(ROOT, "tests", "test_oracle_pins.py")
    r = subprocess.run([sys.executable, "-c", _RUNNER.format(root=ROOT, mutant=str(copy), pins=pins)],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-800:]
