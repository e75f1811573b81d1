"""Do the pins notice a broken oracle?  Each case plants one plausible mistake (a wrong sign, a
swapped index, a dropped term, a transposed role) in a COPY of the oracle's C source, builds
it, and runs the pin tests against that copy in a child process: they must fail.  Everything
here runs on the CPU; the GPU library is not involved."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pdelta_oracle.c")

# (name, text in the oracle, replacement, pin files that must catch it)
MUTATIONS = [
    ("sign of zero becomes -1", "if (!(wf < wb)) B_packed", "if (wf > wb) B_packed", ["test_oracle_pack.py"]),
    ("bits packed MSB first", "|= (uint32_t)1 << (i % 32);", "|= (uint32_t)1 << (31 - i % 32);", ["test_oracle_pack.py"]),
    ("row mean divided by d_out", "pdelta_ref_rne_f16(s_row / (double)d_in)", "pdelta_ref_rne_f16(s_row / (double)d_out)",
     ["test_oracle_pack.py"]),
    ("column mean divided by d_in", "pdelta_ref_rne_f16(s_col / (double)d_out)", "pdelta_ref_rne_f16(s_col / (double)d_in)",
     ["test_oracle_pack.py"]),
    ("absolute value dropped in the row sum", "s_row += fabs(wf - wb);", "s_row += (wf - wb);", ["test_oracle_pack.py"]),
    ("patch subtracts the delta", "pdelta_ref_decode(W_b[o * d_in + i], w_dtype) + scale * b;",
     "pdelta_ref_decode(W_b[o * d_in + i], w_dtype) - scale * b;", ["test_oracle_pack.py", "test_oracle_linear.py"]),
    ("patch indexes the column scale by the row", "double scale = decode_f16(axis == 0 ? v[o] : v[i]);\n            W_hat",
     "double scale = decode_f16(axis == 0 ? v[o] : v[o % d_in]);\n            W_hat", ["test_oracle_linear.py"]),
    ("linear reads X transposed", "acc += Xd[m * d_in + i] * W_hat[o * d_in + i];",
     "acc += Xd[(i % M) * d_in + (m * 7 + i) % d_in] * W_hat[o * d_in + i];", ["test_oracle_linear.py"]),
    ("unpack polarity inverted", "& 1u) ? 1.0 : -1.0;\n    return REF_OK;", "& 1u) ? -1.0 : 1.0;\n    return REF_OK;",
     ["test_oracle_pack.py"]),
    ("fp16 rounding truncates", "uint16_t pdelta_ref_rne_f16(double x)  { return rne_generic(x, 10, -14, 15, 15); }",
     "uint16_t pdelta_ref_rne_f16(double x)  { return rne_generic(x * (1.0 - 1.0 / 4096.0), 10, -14, 15, 15); }",
     ["test_oracle_formats.py"]),
    ("block scale indexed inside the group instead of by the group", "* n_groups + i / group]);",
     "* n_groups + i % n_groups]);", ["test_oracle_group.py"]),
    ("block scale ignores the output row", "return decode_f16(v[(v_rows == 1 ? 0 : o) * n_groups",
     "return decode_f16(v[(v_rows == 1 ? 0 : 0) * n_groups", ["test_oracle_group.py"]),
    ("block mean divided by the group size only", "double count = (double)(o_last - o_first + 1) * (double)group;",
     "double count = (double)group;", ["test_oracle_group.py"]),
    ("gradient modes swapped", "if (axis == 0) {\n                double s = 0.0;", "if (axis == 1) {\n                double s = 0.0;",
     ["test_oracle_linear.py"]),
]


@pytest.mark.parametrize("name,old,new,files", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_the_planted_mistake(name, old, new, files, tmp_path):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"the oracle no longer contains the text this mutation edits: {old!r}"
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(text.replace(old, new, 1))
    mutant_so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(mutant_so),
                    str(mutant_c), "-lm"], check=True)
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          "--oracle-lib", str(mutant_so), *[os.path.join(ROOT, "tests", f) for f in files]],
                         cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert res.returncode != 0, f"no pin noticed: {name}\n{res.stdout[-2000:]}"
    assert " failed" in res.stdout or " error" in res.stdout, res.stdout[-2000:]
