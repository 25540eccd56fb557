"""Do the oracle's pins bite?  Each case plants ONE mistake in a temporary copy of oracle/ivfpq_oracle.c (a
dropped term, a wrong sign or index, a transposed operand, a wrong rounding direction ...), builds that copy
with gcc and runs the oracle's own pin tests (tests/test_oracle_formats.py, tests/test_oracle_ivfpq.py)
against it in a child process: at least one pin must fail.  The tree itself is never modified; nothing here
touches a GPU or the HIP library."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what is planted, text in the source, its replacement)
MUTATIONS = [
    ("per-table bias one binade too high", "else { (void)frexp(mx, &e); e -= 1; }", "else { (void)frexp(mx, &e); }"),
    ("per-table bias with the wrong sign of the exponent", "int bias = ((1 << exp_bits) - 1) - e;", "int bias = ((1 << exp_bits) - 1) + e;"),
    ("largest table entry skips entry 0", "if (!isnan(F[i]) && (double)F[i] > mx) mx = (double)F[i];",
     "if (!isnan(F[i]) && (double)F[i] > mx && i > 0) mx = (double)F[i];"),
    ("per-table bias off by one", "bias = orc_fp8_table_bias(F, n, 8 - mant_bits, bias_min, bias_max);",
     "bias = orc_fp8_table_bias(F, n, 8 - mant_bits, bias_min, bias_max) + 1;"),
    ("truncation that rounds up", "if (truncate) return (uint8_t)lo;", "if (truncate) return (uint8_t)(lo + 1 > 255 ? 255 : lo + 1);"),
    ("re-ranking reads the wrong row", "                if (id < 0) continue;\n                buf[m].key = sqdist_f64(queries + q * d, data + id * d, d);",
     "                if (id < 0) continue;\n                buf[m].key = sqdist_f64(queries + q * d, data + c * d, d);"),
    ("re-ranking drops its first candidate", "                buf[m].id = id;\n                ++m;", "                buf[m].id = id;\n                if (c > 0) ++m;"),
    ("sign of the query residual", "rq[t] = query[t] - centroid[t]", "rq[t] = centroid[t] - query[t]"),
    ("wrong sub-vector index in the table", "float diff = cb[t] - rq[j * m + t]", "float diff = cb[t] - rq[j + t]"),
    ("transposed table index in Eq. (1)", "lut_decoded[(int64_t)j * ksub + code_at(y, j, pq_bits)]",
     "lut_decoded[(int64_t)code_at(y, j, pq_bits) * pq_dim + j]"),
    ("bits of a code read in reverse order", "code |= ((codes[i >> 3] >> (i & 7)) & 1) << b;",
     "code |= ((codes[i >> 3] >> (i & 7)) & 1) << (pq_bits - 1 - b);"),
    ("8-bit encode: ties go down", "(v - table[lo]) >= (table[lo + 1] - v)", "(v - table[lo]) > (table[lo + 1] - v)"),
    ("half encode: ties always up", "if (rem > 0.5 || (rem == 0.5 && (m & 1u))) m += 1;", "if (rem >= 0.5) m += 1;"),
    ("nearest centre: ties to the higher index", "if (dist < best) { best = dist; arg = c; }", "if (dist <= best) { best = dist; arg = c; }"),
    ("Eq. (1) keeps only the last term", "acc = acc + f;", "acc = f;"),
    ("half table without saturation", "if (a > 65504.0) a = 65504.0;", ""),
    ("table entry drops its first component", "acc = fmaf(diff, diff, acc);", "acc = fmaf(diff, diff, acc); if (t == 0 && m > 1) acc = 0.0f;"),
    ("last vector of a cluster not scanned", "int64_t lo = list_offsets[l], len = list_offsets[l + 1] - lo;",
     "int64_t lo = list_offsets[l], len = list_offsets[l + 1] - lo; if (len > 3) len -= 1;"),
    ("ids taken from the wrong cluster", "cand[at].id = ids[lo + i]", "cand[at].id = ids[i]"),
    ("equal distances ordered by descending id",
     "if (x->id < y->id) return -1;\n    if (x->id > y->id) return 1;\n    return 0;\n}\nstatic int cmp_pair_f",
     "if (x->id < y->id) return 1;\n    if (x->id > y->id) return -1;\n    return 0;\n}\nstatic int cmp_pair_f"),
    ("8-bit value one binade too small", "return ldexp(1.0 + (double)m / (double)(1 << mant_bits), e - bias);",
     "return ldexp(1.0 + (double)m / (double)(1 << mant_bits), e - bias - 1);"),
    ("every table built against the nearest probe's centroid", "orc_lut_f32(qv, centroids + (int64_t)l * d,",
     "orc_lut_f32(qv, centroids + (int64_t)probes[0] * d,"),
]


def _copy_tree(dst):
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(dst, "oracle"),
                    ignore=shutil.ignore_patterns("__pycache__", "*.so"))
    os.makedirs(os.path.join(dst, "tests"))
    for name in ("conftest.py", "util_parity.py", "test_oracle_formats.py", "test_oracle_ivfpq.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), os.path.join(dst, "tests", name))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(dst, "tests", "golden"))
    shutil.copy(os.path.join(ROOT, "synth_inputs.py"), os.path.join(dst, "synth_inputs.py"))


def _run_pins(tree):
    env = dict(os.environ, PYTHONPATH=tree, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(tree, "tests", "test_oracle_formats.py"),
                           os.path.join(tree, "tests", "test_oracle_ivfpq.py")],
                          cwd=tree, env=env, capture_output=True, text=True, timeout=600)


def test_unmodified_copy_passes_its_pins(tmp_path):
    # the harness itself: a plain copy of the oracle builds and passes (so a failure below is the mutation's)
    tree = str(tmp_path)
    _copy_tree(tree)
    r = _run_pins(tree)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_fails_a_pin(tmp_path, what, old, new):
    tree = str(tmp_path)
    _copy_tree(tree)
    src = os.path.join(tree, "oracle", "ivfpq_oracle.c")
    text = open(src).read()
    assert text.count(old) >= 1, f"the oracle no longer contains the line this case patches: {old!r}"
    open(src, "w").write(text.replace(old, new, 1))
    r = _run_pins(tree)
    assert r.returncode != 0, f"no pin noticed: {what}"
    assert "failed" in r.stdout or "error" in r.stdout.lower(), r.stdout[-1500:]
