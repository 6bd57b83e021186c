"""Shows that the oracle's pins have teeth: each plausible slip, planted in a
copy of the oracle's source and built on the CPU, must make the pin suite fail.
The mistakes live only in temporary copies; nothing here touches the GPU."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "star_oracle.c")

MUTANTS = [
    ("sum_instead_of_mean", "return a / (double)y;", "return a;"),
    ("decay_sign", "double d = gbar + wd * params[j];", "double d = gbar - wd * params[j];"),
    ("momentum_sign", "momentum[j] = mu * momentum[j] + d;", "momentum[j] = mu * momentum[j] - d;"),
    ("step_sign", "params[j] = params[j] - lr * momentum[j];", "params[j] = params[j] + lr * momentum[j];"),
    ("step_uses_d_not_v", "params[j] = params[j] - lr * momentum[j];", "params[j] = params[j] - lr * d;"),
    ("momentum_dropped", "momentum[j] = mu * momentum[j] + d;", "momentum[j] = d;"),
    ("staleness_off_by_one", "a = 1.0 / (1.0 + (double)up->staleness[idx]);",
     "a = 1.0 / (2.0 + (double)up->staleness[idx]);"),
    ("lr_scale_inverted", "lr *= (double)y / (double)W;", "lr *= (double)W / (double)y;"),
    ("row_index_is_position", "grad_at(rows[up->members[lo + m]], grad_dtype, j)", "grad_at(rows[m], grad_dtype, j)"),
    ("coef_of_first_member", "member_coef(up, hp->wmode, lo + m, y)", "member_coef(up, hp->wmode, lo, y)"),
    ("norm_not_rooted", "norms_out[u] = sqrt(sumsq);", "norms_out[u] = sumsq;"),
    ("norm_after_decay", "sumsq += gbar * gbar;\n            double d = gbar + wd * params[j];",
     "double d = gbar + wd * params[j];\n            sumsq += d * d;"),
    ("bf16_shift", "<< 16; /* bf16", "<< 15; /* bf16"),
    ("lr_of_first_update", "(double)up->lr[u]", "(double)up->lr[0]"),
    ("reduce_output_row_index", "out[(int64_t)u * P + j] = gbar;", "out[j] = gbar;"),
    ("gram_uses_one_row_twice", "s += grad_at(rows[a], grad_dtype, j) * grad_at(rows[b], grad_dtype, j);",
     "s += grad_at(rows[a], grad_dtype, j) * grad_at(rows[a], grad_dtype, j);"),
    ("gram_transposed_store", "out[(int64_t)a * W + b] = s;", "out[(int64_t)a * W + b] = (a <= b) ? s : 0.0;"),
    ("decay_after_step", "double d = gbar + wd * params[j];\n            momentum[j] = mu * momentum[j] + d;\n            params[j] = params[j] - lr * momentum[j];",
     "momentum[j] = mu * momentum[j] + gbar;\n            params[j] = params[j] - lr * momentum[j];\n            params[j] = params[j] - lr * wd * params[j];"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, name, old, new):
    src = open(SRC).read()
    assert old in src, f"mutant {name} no longer matches the oracle's source"
    mutated = src.replace(old, new)
    c = tmp_path / "mut.c"
    c.write_text(mutated)
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-w",
                           "-o", str(lib), str(c), "-lm"])
    env = dict(os.environ, STAR_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 1, f"pins did not notice mutant {name}:\n{r.stdout[-2000:]}"
