"""The pins must be able to fail: each case plants one plausible mistake in a COPY of the
oracle's C source (on the CPU, never in the product), rebuilds it, and requires that at least
one pin test of the matching suite rejects it."""
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "aride_oracle.c")

import test_oracle_actor as t_actor          # noqa: E402
import test_oracle_replay as t_replay        # noqa: E402
import test_oracle_retrace as t_retrace      # noqa: E402
import test_oracle_scan_variants as t_scan   # noqa: E402
import test_oracle_score as t_score          # noqa: E402

# (name, text to find, replacement, pin module)
MUTANTS = [
    ("entropy sign", "if (p > 0.0) ent -= p * logp;", "if (p > 0.0) ent += p * logp;", t_score),
    ("log-sum-exp without the max", "double L = m + log(sum);\n        double ent = 0.0;\n        for (int64_t v = 0; v < V; ++v) {\n            double logp = bf16_to_double(row[v]) - L;\n            double p = exp(logp);\n            if (p > 0.0) ent -= p * logp;",
     "double L = log(sum);\n        double ent = 0.0;\n        for (int64_t v = 0; v < V; ++v) {\n            double logp = bf16_to_double(row[v]) - L;\n            double p = exp(logp);\n            if (p > 0.0) ent -= p * logp;", t_score),
    ("token off by one", "lp[r] = bf16_to_double(row[tok]) - L;", "lp[r] = bf16_to_double(row[tok > 0 ? tok - 1 : 0]) - L;", t_score),
    ("step sum skips a row", "for (int32_t j = 0; j < A; ++j) { sl += lp[n * A + j]; se += en[n * A + j]; }",
     "for (int32_t j = 1; j < A; ++j) { sl += lp[n * A + j]; se += en[n * A + j]; }", t_score),
    ("retrace uses the step's own ratio", "double Delta = (t == hi - 1) ? delta : delta + gamma * c_next * Delta_next;\n            if (target) target[t] = q_t + Delta;\n            if (td) td[t] = delta;\n            if (rho) rho[t] = rho_t;\n            Delta_next = Delta;\n            c_next = lambda * (rho_t < 1.0 ? rho_t : 1.0);",
     "double c_own = lambda * (rho_t < 1.0 ? rho_t : 1.0);\n            double Delta = (t == hi - 1) ? delta : delta + gamma * c_own * Delta_next;\n            if (target) target[t] = q_t + Delta;\n            if (td) td[t] = delta;\n            if (rho) rho[t] = rho_t;\n            Delta_next = Delta;\n            c_next = c_own;", t_retrace),
    ("retrace drops gamma in the trace", "delta + gamma * c_next * Delta_next;", "delta + c_next * Delta_next;", t_retrace),
    ("retrace does not truncate", "c_next = lambda * (rho_t < 1.0 ? rho_t : 1.0);", "c_next = lambda * rho_t;", t_retrace),
    ("retrace ratio inverted", "double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double Delta = (t == hi - 1)", "double rho_t = exp(logp_mu[t] - logp_pi[t]);\n            double Delta = (t == hi - 1)", t_retrace),
    ("TD error sign of V", "double delta = reward[t] + gamma * v_next - q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double Delta = (t == hi - 1)",
     "double delta = reward[t] + gamma * v_next + q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double Delta = (t == hi - 1)", t_retrace),
    ("bootstrap ignored", "double v_next = (t == hi - 1) ? (boot ? boot[b] : 0.0) : value[t + 1];\n            double q_t = q ? q[t] : value[t];\n            double delta = reward[t] + gamma * v_next - q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double Delta = (t == hi - 1)",
     "double v_next = (t == hi - 1) ? 0.0 : value[t + 1];\n            double q_t = q ? q[t] : value[t];\n            double delta = reward[t] + gamma * v_next - q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double Delta = (t == hi - 1)", t_retrace),
    ("priority forgets the absolute value", "w_td * fabs(td[t]) / td_scale", "w_td * td[t] / td_scale", t_replay),
    ("priority mean divides by B", "acc / (double)(hi - lo)", "acc / (double)B", t_replay),
    ("update keeps the first duplicate", "weights[idx[k]] = (float)pow(p, (double)alpha);", "if (weights[idx[k]] == 0.0f) weights[idx[k]] = (float)pow(p, (double)alpha);", t_replay),
    ("sampler uses >= instead of >", "if (C[mid] > t) hi = mid; else lo = mid + 1;", "if (C[mid] >= t) hi = mid; else lo = mid + 1;", t_replay),
    ("quantisation rounds instead of floors", "qi = (uint64_t)floor(ldexp(w, 39 - e));", "qi = (uint64_t)floor(ldexp(w, 39 - e) + 0.5);", t_replay),
    ("exponent off by one", "int e = ilogb(wmax) + 1;", "int e = ilogb(wmax);", t_replay),
    ("circular index does not wrap", "i = (i + 1) % M;", "i = (i + 1) < M ? (i + 1) : M - 1;", t_replay),
    ("actor gradient drops the one-hot", "double onehot = (v == tok) ? 1.0 : 0.0;", "double onehot = 0.0;", t_actor),
    ("actor entropy gradient sign", "grad[r * V + v] = scale * (-coef * (onehot - p) + beta * ent_term);", "grad[r * V + v] = scale * (-coef * (onehot - p) - beta * ent_term);", t_actor),
    ("actor loss forgets the entropy bonus", "loss += -coef * step_logp - beta * step_ent +", "loss += -coef * step_logp +", t_actor),
    ("v-trace weights the TD error with the unclipped ratio", "double Delta = rho_clip * delta +", "double Delta = rho_t * delta +", t_scan),
    ("v-trace uses the next step's coefficient", "gamma * c_t * Delta_next);\n            if (target) target[t] = q_t + Delta;\n            if (td) td[t] = delta;\n            if (rho) rho[t] = rho_t;\n            Delta_next = Delta;\n        }",
     "gamma * c_prev * Delta_next);\n            if (target) target[t] = q_t + Delta;\n            if (td) td[t] = delta;\n            if (rho) rho[t] = rho_t;\n            Delta_next = Delta;\n            c_prev = c_t;\n        }", t_scan),
    ("monte-carlo return without discount", "G = reward[t] + gamma * G;", "G = reward[t] + G;", t_scan),
]


def _load_mutant(tmp_path, name, find, repl):
    src = open(SRC).read()
    assert src.count(find) >= 1, f"mutant '{name}': pattern not found in the oracle source"
    mutated = src.replace(find, repl, 1)
    if "c_prev" in repl and "double c_prev" not in mutated:
        mutated = mutated.replace("double Delta_next = 0.0;\n        for (int64_t t = hi - 1; t >= lo; --t) {\n            double v_next = (t == hi - 1) ? (boot ? boot[b] : 0.0) : value[t + 1];\n            double q_t = q ? q[t] : value[t];\n            double delta = reward[t] + gamma * v_next - q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double rho_clip",
                                  "double Delta_next = 0.0, c_prev = 0.0;\n        for (int64_t t = hi - 1; t >= lo; --t) {\n            double v_next = (t == hi - 1) ? (boot ? boot[b] : 0.0) : value[t + 1];\n            double q_t = q ? q[t] : value[t];\n            double delta = reward[t] + gamma * v_next - q_t;\n            double rho_t = exp(logp_pi[t] - logp_mu[t]);\n            double rho_clip", 1)
    c_path = tmp_path / "mutant.c"
    so_path = tmp_path / "libmutant.so"
    c_path.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(so_path),
                    str(c_path), "-lm"], check=True)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{abs(hash(name))}",
                                                  os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._LIB_PATH = str(so_path)
    mod._lib = None
    mod._load()
    return mod


def _pins_of(module):
    out = []
    for name in sorted(dir(module)):
        fn = getattr(module, name)
        if name.startswith("test_") and callable(fn) and "oracle" in fn.__code__.co_varnames[:fn.__code__.co_argcount]:
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                out.append((name, fn, [{}]))
            else:
                m = marks[0]
                keys = [k.strip() for k in m.args[0].split(",")]
                cases = [dict(zip(keys, v if isinstance(v, (tuple, list)) and len(keys) > 1 else (v,))) for v in m.args[1]]
                out.append((name, fn, cases))
    return out


@pytest.mark.parametrize("name,find,repl,suite", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, find, repl, suite):
    mutant = _load_mutant(tmp_path, name, find, repl)
    caught = []
    for tname, fn, cases in _pins_of(suite):
        for kw in cases:
            try:
                fn(mutant, **kw)
            except (AssertionError, ValueError, ZeroDivisionError, IndexError) as exc:
                caught.append(f"{tname}: {type(exc).__name__}")
                break
    assert caught, f"no pin noticed the planted mistake '{name}'"


def test_the_unmodified_oracle_passes_the_same_harness(tmp_path):
    # guards the harness itself: with no mistake planted, no pin may fire
    mod = _load_mutant(tmp_path, "identity", "double L = m + log(sum);", "double L = m + log(sum);")
    for suite in (t_score, t_retrace, t_replay, t_actor, t_scan):
        for tname, fn, cases in _pins_of(suite):
            for kw in cases:
                fn(mod, **kw)
