"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle's C source
(a dropped term, a wrong sign or index, an inverted mask, a wrong rounding rule), builds it on the
CPU, runs the pin tests against the mutated library and requires at least one of them to fail.
The real oracle is untouched; nothing here runs on a GPU."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
from paper_2504_04673_amd import synth
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "sagnn_oracle.c")


def cfg1_inputs():
    return synth.er_graph(4096, 8, 0), synth.uniform((4096, 16), 0, synth.STREAM_H)


def spmm_pins():
    pins.test_spmm_bruteforce_dense(7, 5, 3, 1)
    pins.test_spmm_bruteforce_dense(33, 64, 17, 2)
    pins.test_spmm_identity_bit_exact()
    pins.test_spmm_regular_ring_all_ones(101, 6, 5)
    pins.test_spmm_accumulate_adds_old_value()


def plan_pins():
    pins.test_needed_rows_bruteforce(1, 25, 64, 4)
    pins.test_needed_rows_bruteforce(2, 40, 130, 7)
    pins.test_needed_rows_empty_and_full()


def pack_pins():
    pins.test_pack_rows_is_fancy_indexing(cfg1_inputs())


def gemm_pins():
    for tx, tw in ((False, False), (False, True), (True, False)):
        pins.test_gemm_vs_numpy_fp64(5, 7, 3, tx, tw)
    pins.test_bf16_round_known_values_and_torch()
    pins.test_gemm_bf16_rounds_operands()


def magnitude_pins():
    for tx, tw in ((False, False), (False, True), (True, False), (True, True)):
        pins.test_gemm_magnitude_companion_with_given_scale(tx, tw)
    pins.test_layer_magnitude_companions_propagate_the_spmm_scale()


def layer_pins():
    pins.test_gcn_layer_fwd_against_dense_numpy()
    pins.test_gcn_backward_finite_differences()


MUTANTS = [
    # (name, text in the source, replacement, pins that must catch it)
    ("spmm drops the old value when accumulating",
     "s[c] = accumulate ? (double)C[r * ldc + c] : 0.0;", "s[c] = 0.0;", spmm_pins),
    ("spmm multiplies every entry of a row by the row of B of its first entry",
     "const float* brow = B + (int64_t)colidx[e] * ldb;",
     "const float* brow = B + (int64_t)colidx[rowptr[r]] * ldb;", spmm_pins),
    ("spmm drops the last entry of every row",
     "for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) {   /* stored order */",
     "for (int64_t e = rowptr[r]; e < rowptr[r + 1] - 1; ++e) {", spmm_pins),
    ("spmm subtracts", "          s[c] += t;", "          s[c] -= t;", spmm_pins),
    ("spmm magnitude companion sums signed terms", "a[c] += fabs(t);", "a[c] += t;", spmm_pins),
    ("needed rows: block offsets shifted by one", "    blk_off[q] = N;", "    blk_off[q] = N + (q > 0);",
     plan_pins),
    ("needed rows: compact index is the original column", "compact[e] = pos[colidx[e]];",
     "compact[e] = colidx[e];", plan_pins),
    ("needed rows: a stored entry with column 0 is forgotten", "    flag[c] = 1;", "    flag[c] = (c != 0);",
     plan_pins),
    ("pack copies row r instead of rows[r]", "H + (int64_t)rows[r] * ldh", "H + (int64_t)r * ldh", pack_pins),
    ("gemm rounds only one operand to bfloat16", "if (bf16) { x = bf16_round(x); w = bf16_round(w); }",
     "if (bf16) { x = bf16_round(x); }", gemm_pins),
    ("bfloat16 rounds ties up instead of to even", "u += 0x7FFFu + lsb;", "u += 0x8000u;", gemm_pins),
    ("gemm skips the last term of every sum", "for (int64_t p = 0; p < k; ++p) {",
     "for (int64_t p = 0; p + 1 < k || (p == 0 && k == 1); ++p) {", gemm_pins),
    ("forward ReLU mask inverted", "(act == 1 && !(Z[i] > 0.0f)) ? 0.0f : Z[i]",
     "(act == 1 && (Z[i] > 0.0f)) ? 0.0f : Z[i]", layer_pins),
    ("backward ReLU mask inverted", "if (!(Zprev[i] > 0.0f)) Gprev[i] = 0.0f;",
     "if (Zprev[i] > 0.0f) Gprev[i] = 0.0f;", layer_pins),
    ("weight gradient uses G instead of A*G",
     "oracle_gemm(Hprev, f_in, 1, S, f_out, 0, f_in, m, f_out, bf16, Y, f_out, NULL, Yabs);",
     "oracle_gemm(Hprev, f_in, 1, G, f_out, 0, f_in, m, f_out, bf16, Y, f_out, NULL, Yabs);", layer_pins),
    ("layer forward multiplies before aggregating with the wrong operand order kept: T is H",
     "oracle_spmm(rowptr, colidx, val, m, H, ldh, f_in, T, f_in, 0, Tabs);\n  oracle_gemm(T,",
     "oracle_spmm(rowptr, colidx, val, m, H, ldh, f_in, T, f_in, 0, Tabs);\n  oracle_gemm(H,", layer_pins),
    ("gemm magnitude ignores the scale handed down from the earlier product",
     "double xa = Xabs ? (transX ? Xabs[p * m + i] : Xabs[i * k + p]) : fabs((double)x);",
     "double xa = fabs((double)x);", magnitude_pins),
    ("gemm magnitude reads the handed-down scale untransposed",
     "(transX ? Xabs[p * m + i] : Xabs[i * k + p])", "Xabs[i * k + p]", magnitude_pins),
    ("gemm magnitude multiplies by signed weights", "a += xa * fabs((double)w);", "a += xa * (double)w;",
     magnitude_pins),
    ("layer forward does not hand the SpMM scale to the GEMM", "bf16, Z, f_out, Tabs, Zabs);",
     "bf16, Z, f_out, NULL, Zabs);", magnitude_pins),
    ("layer backward does not hand the SpMM scale to the GEMM", "Gprev, f_in, Sabs, Gabs);",
     "Gprev, f_in, NULL, Gabs);", magnitude_pins),
]


@pytest.mark.parametrize("name,old,new,run_pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(name, old, new, run_pins, monkeypatch):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site not unique: {old!r}"
    with tempfile.TemporaryDirectory() as tmp:
        c_path, so_path = os.path.join(tmp, "mutant.c"), os.path.join(tmp, "mutant.so")
        open(c_path, "w").write(src.replace(old, new))
        subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-o", so_path,
                        c_path, "-lm"], check=True)
        monkeypatch.setattr(oracle, "_lib", oracle._declare(ctypes.CDLL(so_path)))
        with pytest.raises((AssertionError, IndexError, ValueError)):
            run_pins()
    monkeypatch.undo()
    run_pins()          # and the unmutated oracle passes the same pins
