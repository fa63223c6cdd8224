"""Do the oracle's pins notice a plausible mistake?  Each case below plants one in a copy of
oracle/kvp_oracle.c (a wrong sign, a wrong index, an off-by-one, a missing factor, a transposed
role), builds it, and runs tests/test_oracle_pins.py against it in a child process: the pins must
fail.  The mistakes are planted in the oracle, on the CPU; the HIP path is not involved.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvp_oracle.c")

MUTANTS = [
    ("theta exponent loses its factor 2", "-2.0 * (double)i / (double)d", "-1.0 * (double)i / (double)d"),
    ("angle of position pos + 1", "double a = (double)pos * (double)inv_freq[i];", "double a = (double)(pos + 1) * (double)inv_freq[i];"),
    ("rotation: wrong sign in the first row", "float lo = xc - ys;", "float lo = xc + ys;"),
    ("rotation: wrong sign in the second row", "float hi = yc + xs;", "float hi = yc - xs;"),
    ("rotation: cos and sin exchanged", "volatile float xc = x[i] * c[i];", "volatile float xc = x[i] * s[i];"),
    ("rotation pairs neighbours instead of i with i + d/2", "volatile float ys = x[i + h] * s[i];", "volatile float ys = x[i ^ 1] * s[i];"),
    ("fused multiply-add instead of separately rounded products", "float lo = xc - ys;", "float lo = __builtin_fmaf(x[i], c[i], -ys);"),
    ("subnormal results flushed to zero", "float lo = xc - ys;", "float lo = xc - ys; if (lo < 1.17549435e-38f && lo > -1.17549435e-38f) lo = 0.f;"),
    ("bf16 store truncates", "u += 0x7FFFu + lsb;", "u += 0u * lsb;"),
    ("bf16 store rounds half up", "u += 0x7FFFu + lsb;", "u += 0x8000u + 0u * lsb;"),
    ("offsets overlap by a row per packet", "        delta += len;\n", "        delta += len > 1 ? len - 1 : len;\n"),
    ("every packet rotated by base_pos", "        kvo_cos_sin(delta, inv_freq, d, c, s);\n#pragma omp parallel for collapse(2) schedule(static)", "        kvo_cos_sin(base_pos, inv_freq, d, c, s);\n#pragma omp parallel for collapse(2) schedule(static)"),
    ("values rotated like keys", "                memcpy((char *)v_out + dst0 * es,\n                       (const char *)pk_v[j] + src0 * es, (size_t)len * d * es);", "                for (int t = 0; t < len; ++t) {\n                    for (int e = 0; e < d; ++e) x[e] = load_elem(pk_v[j], dtype, src0 + (size_t)t * d + e);\n                    kvo_rotate(x, d, c, s, y);\n                    for (int e = 0; e < d; ++e) store_elem(v_out, dtype, dst0 + (size_t)t * d + e, y[e]);\n                }"),
    ("query one position late", "int64_t pos = ctx_len + t;", "int64_t pos = ctx_len + t + 1 < t_cap ? ctx_len + t + 1 : ctx_len + t;"),
    ("query token does not see itself", "int64_t n_vis = ctx_len + t + 1;", "int64_t n_vis = ctx_len + t;"),
    ("query token sees the next one", "int64_t n_vis = ctx_len + t + 1;", "int64_t n_vis = ctx_len + t + 2 < t_cap ? ctx_len + t + 2 : t_cap;"),
    ("query heads dealt round-robin to kv heads", "int h = hq / g;", "int h = hq % n_kv;"),
    ("scores divided by d", "double scale = 1.0 / sqrt((double)d);", "double scale = 1.0 / (double)d;"),
    ("scores not scaled", "double scale = 1.0 / sqrt((double)d);", "double scale = 1.0;"),
    ("softmax not normalised", "o[e] /= denom;", "o[e] /= 1.0;"),
    ("pruned packets advance positions by their kept rows", "        delta += spans[j];\n", "        delta += rows[j];\n"),
    ("pruned packets overlap by a row each", "        row0 += rows[j];\n", "        row0 += rows[j] > 1 ? rows[j] - 1 : rows[j];\n"),
    ("pruned path: query rotated by its row, not its position", "kvo_cos_sin(pos0 + t, inv_freq, d, c, s);", "kvo_cos_sin(row0 + t, inv_freq, d, c, s);"),
]



def run_pins_against(lib):
    """Runs the pins in a child process whose oracle is `lib`.  The oracle front end takes another
    library only when both variables are set (the second one names this test as the one asking),
    and says so on stderr.  Every planted mistake keeps its accesses in bounds, so the child ends;
    the time limit is there so that a child that does not is reported instead of waited for."""
    env = dict(os.environ, KVP_ORACLE_LIB=str(lib), KVP_ORACLE_LIB_FOR="tests/test_oracle_mutants.py")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_the_pins(tmp_path, what, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, "the oracle no longer contains: " + old
    mutated = tmp_path / "kvp_oracle_mutant.c"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / "libkvp_oracle_mutant.so"
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", str(lib),
                    str(mutated), "-lm"], check=True)
    r = run_pins_against(lib)
    # (a pin that fails, or a child that dies on an out-of-range row: either way it was noticed)
    assert r.returncode != 0, "the pins passed with this mistake planted: %s\n%s" % (what, r.stdout[-2000:])


def test_the_unmodified_oracle_passes_through_the_same_route(tmp_path):
    lib = tmp_path / "libkvp_oracle_copy.so"
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), SRC, "-lm"],
                   check=True)
    r = run_pins_against(lib)
    assert r.returncode == 0, r.stdout[-2000:]
