"""Planted mistakes: build broken copies of the oracle's C source and check that the pin suite
notices each one.  A mistake is planted in the oracle only, on the CPU; nothing here touches
the GPU path.  This shows the pins are strong enough that a dropped term, a wrong sign or
index, a transposed operand or a lost scale would not go unnoticed."""
import os
import subprocess

import pytest

import oracle
import oracle_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "csr_oracle.c")

# (name, text to find, replacement, which occurrence (0-based) to replace)
MUTANTS = [
    ("spmm_drops_vals", "const double s = (double)vals[j];", "const double s = 1.0;", 0),
    ("spmm_sign", "acc[l] += term;", "acc[l] -= term;", 0),
    ("spmm_reversed_columns", "const double term = s * (double)Bk[l];",
     "const double term = s * (double)Bk[N - 1 - l];", 0),
    ("spmm_drops_last_entry", "for (int32_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {\n            const double s",
     "for (int32_t j = rowptr[i]; j < rowptr[i + 1] - 1; ++j) {\n            const double s", 0),
    ("spmm_skips_first_entry", "for (int32_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {\n            const double s",
     "for (int32_t j = rowptr[i] + 1; j < rowptr[i + 1]; ++j) {\n            const double s", 0),
    ("spmm_same_column_for_all", "const int32_t k = colidx[j];\n            const float *Bk = B + (size_t)k * N;",
     "const int32_t k = colidx[rowptr[i]];\n            const float *Bk = B + (size_t)k * N;", 0),
    ("spmm_abs_sum_signed", "aac[l] += fabs(term);", "aac[l] += term;", 0),
    ("spmm_ignores_row_list", "const int32_t i = rows ? rows[t] : t;", "const int32_t i = t;", 0),
    ("sddmm_ignores_row_list", "const int32_t i = rows ? rows[t] : t;", "const int32_t i = t;", 1),
    ("fused_ignores_row_list", "const int32_t i = rows ? rows[t] : t;", "const int32_t i = t;", 2),
    ("sddmm_reversed_A", "const double term = (double)Ai[l] * (double)Bk[l];",
     "const double term = (double)Ai[D - 1 - l] * (double)Bk[l];", 0),
    ("sddmm_short_dot", "for (int32_t l = 0; l < D; ++l) {", "for (int32_t l = 0; l < D - 1; ++l) {", 0),
    ("sddmm_drops_scale", "P[j] = s * dp;", "P[j] = dp;", 0),
    ("sddmm_abs_scale", "P[j] = s * dp;", "P[j] = fabs(s) * dp;", 0),
    ("sddmm_fp32_accumulate", "double dp = 0.0, adp = 0.0;", "float dp = 0.0f; double adp = 0.0;", 0),
    ("sddmm_wrong_B_row", "const int32_t k = colidx[j];\n            const float *Bk = B + (size_t)k * D;",
     "const int32_t k = colidx[rowptr[i]];\n            const float *Bk = B + (size_t)k * D;", 0),
    ("fused_reversed_A", "const double term = (double)Ai[l] * (double)Bk[l];",
     "const double term = (double)Ai[D - 1 - l] * (double)Bk[l];", 1),
    ("fused_drops_scale", "arow[j] = s * dp;", "arow[j] = dp;", 0),
    ("fused_rounds_scores_to_fp32", "arow[j] = s * dp;", "arow[j] = (double)(float)(s * dp);", 0),
    ("fused_second_stage_wrong_row", "const float *Ck = C + (size_t)k * N;",
     "const float *Ck = C + (size_t)colidx[rowptr[i]] * N;", 0),
    ("fused_second_stage_sign", "acc[l] += arow[j] * (double)Ck[l];", "acc[l] -= arow[j] * (double)Ck[l];", 0),
    ("fused_abs_sum_unscaled", "aabs[j] = fabs(s) * adp;", "aabs[j] = adp;", 0),
    ("fused_skips_last_score", "for (int32_t j = 0; j < nnzr; ++j) {\n            const int32_t k = colidx[rowptr[i] + j];\n            const float *Ck",
     "for (int32_t j = 0; j < nnzr - 1; ++j) {\n            const int32_t k = colidx[rowptr[i] + j];\n            const float *Ck", 0),
]


def _replace_nth(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, f"mutation site not found: {old!r} (occurrence {n})"
    return text[:pos] + new + text[pos + len(old):]


@pytest.mark.parametrize("name,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, nth, tmp_path, monkeypatch):
    src = _replace_nth(open(SRC).read(), old, new, nth)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", str(c), "-o", str(so), "-lm"],
                   check=True)
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", oracle._bind(str(so)))
    caught = []
    for pin in oracle_pins.PINS:
        try:
            pin()
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin noticed the planted mistake {name!r}"
