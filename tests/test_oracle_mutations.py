"""Plants one mistake at a time in a COPY of the oracle's C source (dropped term, wrong
sign, wrong index, dropped factor, narrower accumulator ...) and checks that the pins fail
for every such copy - and pass for the unmodified source.  CPU only."""
import os
import subprocess

import pytest

import _pins_core

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "distal_oracle.c")

# (name, text to find exactly once, replacement) - every mutant stays inside its arrays
MUTATIONS = [
    ("gemm_sign", "s += ld_elem(A, dt, i * lda + k) * ld_elem(B, dt, k * ldb + j);",
     "s -= ld_elem(A, dt, i * lda + k) * ld_elem(B, dt, k * ldb + j);"),
    ("gemm_dropped_term", "for (int64_t k = 0; k < K; ++k)\n                s += ld_elem(A, dt, i * lda + k)",
     "for (int64_t k = 0; k < K - 1; ++k)\n                s += ld_elem(A, dt, i * lda + k)"),
    ("gemm_dropped_init", "if (accumulate) s = ld_elem(init, dt, i * ldinit + j) + s;", "if (accumulate) s = s;"),
    ("gemm_wrong_column", "ld_elem(B, dt, k * ldb + j);", "ld_elem(B, dt, k * ldb + (N - 1 - j));"),
    ("gemm_ignores_lda", "ld_elem(A, dt, i * lda + k)", "ld_elem(A, dt, i * K + k)"),
    ("gemm_ignores_ldb", "ld_elem(B, dt, k * ldb + j);", "ld_elem(B, dt, k * N + j);"),
    ("ttv_wrong_index", "\n                s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, k);",
     "\n                s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(c, dt, K - 1 - k);"),
    ("innerprod_dropped_tail", "for (int64_t m = lo; m < hi; ++m)", "for (int64_t m = lo; m < hi - 1; ++m)"),
    ("innerprod_wrong_pairing", "ld_elem(B, dt, m) * ld_elem(C, dt, m);", "ld_elem(B, dt, m) * ld_elem(C, dt, lo + hi - 1 - m);"),
    ("ttm_wrong_column", "ld_elem(C, dt, k * L + l);", "ld_elem(C, dt, k * L + (L - 1 - l));"),
    ("mttkrp_dropped_factor", "\n                         * ld_elem(D, dt, k * L + l);", ";"),
    ("mttkrp_swapped_factor_rows", "ld_elem(C, dt, j * L + l)\n                         *",
     "ld_elem(C, dt, (J - 1 - j) * L + l)\n                         *"),
    ("ttm_mode0_transposed_factor", "ld_elem(C, dt, i * R + r);", "ld_elem(C, dt, r * I + i);"),
    ("ttm_mode1_output_misplaced", "out[(i * R + r) * K + k] = (double)s;", "out[(i * K + k) * R + r] = (double)s;"),
    ("ttm_mode1_dropped_term", "for (int64_t j = 0; j < J; ++j)\n                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, j * R + r);",
     "for (int64_t j = 1; j < J; ++j)\n                        s += ld_elem(B, dt, (i * J + j) * K + k) * ld_elem(C, dt, j * R + r);"),
    ("mttkrp_mode1_dropped_term", "for (int64_t i = 0; i < I; ++i)\n                    for (int64_t k = 0; k < K; ++k)",
     "for (int64_t i = 0; i < I - 1; ++i)\n                    for (int64_t k = 0; k < K; ++k)"),
    ("mttkrp_mode1_dropped_factor", "ld_elem(C, dt, i * L + l)\n                             * ld_elem(D, dt, k * L + l);",
     "ld_elem(C, dt, i * L + l);"),
    ("mttkrp_mode2_swapped_factor_rows", "ld_elem(D, dt, j * L + l);", "ld_elem(D, dt, (J - 1 - j) * L + l);"),
    ("mttkrp_mode2_output_transposed", "out[k * L + l] = (double)s;", "out[l * K + k] = (double)s;"),
    ("ttv_mode0_wrong_weight", "ld_elem(c, dt, i);", "ld_elem(c, dt, I - 1 - i);"),
    ("ttv_mode1_output_transposed", "out[i * K + k] = (double)s;", "out[k * I + i] = (double)s;"),
    ("narrow_accumulator", "typedef long double acc_t;", "typedef double acc_t;"),
]


def build_variant(tmp_path, name, old, new):
    import oracle
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"{name}: pattern must occur exactly once"
        text = text.replace(old, new)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                           "-o", str(so), str(c)])
    return oracle.Variant(str(so))


def test_pins_pass_on_the_unmodified_source(tmp_path):
    _pins_core.run(build_variant(tmp_path, "clean", None, None))


def test_pins_pass_on_the_installed_oracle(oracle):
    _pins_core.run(oracle)


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    mutant = build_variant(tmp_path, name, old, new)
    with pytest.raises(AssertionError):
        _pins_core.run(mutant)
