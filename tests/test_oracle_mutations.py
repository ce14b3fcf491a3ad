"""Every part of the oracle is pinned: a single planted mistake anywhere in it must make a pin fail.

Each case copies the oracle (and the CPU pin tests with what they import) into a scratch directory, changes ONE
line of the copy of stripe_oracle.c, rebuilds it there and runs the pin tests against the copy in a child
process: the pins must fail.  The un-mutated copy must pass, so a failure is the mutation's doing.  Nothing here
touches the GPU or the HIP library; the repository's own oracle is never modified.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what the slip is, text as it stands, text with the slip)
MUTATIONS = [
    ("constraint test off by one", "if (s < 0) return SO_OK;", "if (s <= 0) return SO_OK;"),
    ("access constant dropped", "int64_t s = ref->access_const[d];", "int64_t s = 0;"),
    ("view check sums only the last level", "for (int m = l + 1; m <= L; ++m) rel += ", "for (int m = l + 1; m <= L; ++m) rel = "),
    ("strides transposed", "addr[r] += c->lvl[l]->refs[r].strides[d] * c->coord[l][r][d];",
     "addr[r] += c->lvl[0]->refs[r].strides[ndim-1-d] * c->coord[l][r][d];"),
    ("root origin left out of the address", "for (int l = 0; l <= L; ++l) addr[r] +=", "for (int l = 1; l <= L; ++l) addr[r] +="),
    ("max compares the wrong way", "case SO_AGG_MAX: if (v > acc) acc = v; break;", "case SO_AGG_MAX: if (v < acc) acc = v; break;"),
    ("min compares the wrong way", "case SO_AGG_MIN: if (v < acc) acc = v; break;", "case SO_AGG_MIN: if (v > acc) acc = v; break;"),
    ("passed constant dropped", "int64_t s = b->passed_const ? b->passed_const[p] : 0;", "int64_t s = 0;"),
    ("passed value ignored", "c->vars[L][b->n_idx + p] = s;", "c->vars[L][b->n_idx + p] = 0;"),
    ("second operand replaced by the first", "v = (leaf->intrinsic == SO_INTR_MUL) ? a * b : a + b;",
     "v = (leaf->intrinsic == SO_INTR_MUL) ? a * a : a + b;"),
    ("bf16 widened with the wrong shift", "uint32_t u = ((uint32_t)h) << 16;", "uint32_t u = ((uint32_t)h) << 15;"),
    ("constraint constant dropped", "int64_t s = b->cons_const[q];", "int64_t s = 0;"),
    ("constraint coefficients read transposed", "s += b->cons_coeff[(size_t)q * nv + v] * c->vars[L][v];",
     "s += b->cons_coeff[(size_t)v * b->n_cons + q] * c->vars[L][v];"),
    ("view containment not checked", "if (rel < 0 || rel >= c->lvl[l]->refs[r].sizes[d])", "if (0)"),
    ("assign conflicts of outer levels not detected", "last / c->iters[l] == ord / c->iters[l] && last != ord", "0"),
    ("first write adds to the prior contents", "      c->touched[e] = 1;\n      c->out_f64[e] = v;", "      c->touched[e] = 1;\n      c->out_f64[e] += v;"),
    ("int8 loaded as unsigned", "return (int64_t)((const int8_t*)base)[addr];", "return (int64_t)((const uint8_t*)base)[addr];"),
    ("relu cut dropped", "if (leaf->intrinsic == SO_INTR_ADD_RELU && v < 0) v = 0;", ";"),
    ("sum aggregation subtracts", "case SO_AGG_ADD: acc = acc + v; break;", "case SO_AGG_ADD: acc = acc - v; break;"),
    ("int32 range of partial sums not checked", "if (!fits_i32(acc)) return fail(", "if (0) return fail("),
]

PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_program_oracle.py", "tests/test_golden_figure5.py"]


def _scratch_copy(tmp_path):
    for d in ("oracle", "tests"):
        shutil.copytree(os.path.join(ROOT, d), tmp_path / d,
                        ignore=shutil.ignore_patterns("*.so", "__pycache__", "test_oracle_mutations.py", "test_gpu*", "test_zz*"))
    os.makedirs(tmp_path / "paper_1903_06498_amd")
    for f in ("__init__.py", "workloads.py"):
        shutil.copy(os.path.join(ROOT, "paper_1903_06498_amd", f), tmp_path / "paper_1903_06498_amd" / f)
    return tmp_path


def _run_pins(where):
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PIN_FILES,
                          cwd=where, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)


def test_unmutated_copy_passes(tmp_path):
    where = _scratch_copy(tmp_path)
    p = _run_pins(where)
    assert p.returncode == 0, p.stdout.decode()[-2000:]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_fails_a_pin(what, old, new, tmp_path):
    where = _scratch_copy(tmp_path)
    src = where / "oracle" / "stripe_oracle.c"
    text = src.read_text()
    assert text.count(old) >= 1, f"mutation '{what}' no longer applies: the oracle's text changed"
    src.write_text(text.replace(old, new))
    p = _run_pins(where)
    assert p.returncode != 0, f"planted mistake survived every pin: {what}"
