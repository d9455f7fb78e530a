"""The pins of test_oracle_pins.py must notice a plausible mistake anywhere in the oracle.  Each case below
plants ONE mistake in a copy of the oracle's source (on the CPU, in a temporary directory), builds it, routes
the pins to that copy and requires at least one of them to fail."""
import os
import shutil
import subprocess

import pytest

import oracle
from tests import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(oracle.__file__))

MUTANTS = {  # name: (file, text to find, replacement)
    "hash modulus 2^31": ("sams_oracle.c", "% 2147483647ULL", "% 2147483648ULL"),
    "sign hash inverted": ("sams_oracle.c", "& 1u) ? -1 : 1", "& 1u) ? 1 : -1"),
    "sketch ignores the sign": ("sams_oracle_impl.h", "REAL term = (sg > 0) ? u[l] : -u[l];", "REAL term = u[l];"),
    "sketch uses the sign hash for the bucket": ("sams_oracle_impl.h",
                                                 "int64_t b = orc_bucket(hp[0], hp[1], (uint32_t)l, c);\n            int sg = orc_sign(hp[2], hp[3], (uint32_t)l);\n            REAL term",
                                                 "int64_t b = orc_bucket(hp[2], hp[3], (uint32_t)l, c);\n            int sg = orc_sign(hp[2], hp[3], (uint32_t)l);\n            REAL term"),
    "aggregate is a sum, not a mean": ("sams_oracle_impl.h", "S_mean[t] = acc / (REAL)n;", "S_mean[t] = acc;"),
    "upper median": ("sams_oracle_impl.h", "REAL med = vals[(r - 1) / 2];", "REAL med = vals[r / 2];"),
    "mean of rows instead of median": ("sams_oracle_impl.h", "REAL med = vals[(r - 1) / 2];",
                                        "REAL med = 0; for (int32_t j = 0; j < r; ++j) med += vals[j] / r;"),
    "unsketch multiplies by sqrt(vhat)": ("sams_oracle_impl.h", "est[t] = vhat ? med / FN(orc_sqrt)(vhat[t]) : med;",
                                          "est[t] = vhat ? med * FN(orc_sqrt)(vhat[t]) : med;"),
    "unsketch divides by vhat": ("sams_oracle_impl.h", "est[t] = vhat ? med / FN(orc_sqrt)(vhat[t]) : med;",
                                 "est[t] = vhat ? med / vhat[t] : med;"),
    "unsketch ignores the sign": ("sams_oracle_impl.h", "vals[j] = (sg > 0) ? q : -q;", "vals[j] = q;"),
    "top-k by signed value": ("sams_oracle_impl.h", "p[l].mag = est[l] < (REAL)0 ? -est[l] : est[l];", "p[l].mag = est[l];"),
    "ties to the larger index": ("sams_oracle_impl.h", "return (a->idx > b->idx) - (a->idx < b->idx);",
                                 "return (a->idx < b->idx) - (a->idx > b->idx);"),
    "refine keeps the coordinates but the wrong values": ("sams_oracle_impl.h", "delta_out[q] = delta_in[pos[q]];", "delta_out[q] = delta_in[q];"),
    "PA: second moment fed with g, not g^2": ("sams_oracle_impl.h", "omb2 * (g[t] * g[t])", "omb2 * g[t]"),
    "PA: scaling by v instead of vhat": ("sams_oracle_impl.h", "e_u[t] = mm / FN(orc_sqrt)(vhat_w[t]) + rho * e_u[t];",
                                         "e_u[t] = mm / FN(orc_sqrt)(vv) + rho * e_u[t];"),
    "PA: error feedback also scaled": ("sams_oracle_impl.h", "e_u[t] = mm / FN(orc_sqrt)(vhat_w[t]) + rho * e_u[t];",
                                       "e_u[t] = (mm + rho * e_u[t]) / FN(orc_sqrt)(vhat_w[t]);"),
    "gather sums instead of averaging": ("sams_oracle_impl.h", "REAL mean = acc / (REAL)n;", "REAL mean = acc;"),
    "gather skips the vhat scaling": ("sams_oracle_impl.h", "delta[q] = vhat ? mean / FN(orc_sqrt)(vhat[l]) : mean;",
                                      "delta[q] = mean;"),
    "beta1 and 1-beta1 swapped": ("sams_oracle_impl.h", "REAL mm = beta1 * m[t] + omb1 * g[t];", "REAL mm = omb1 * m[t] + beta1 * g[t];"),
    "error feedback scaled on m": ("sams_oracle_impl.h", "e_u[t] = mm + rho * e_u[t];", "e_u[t] = rho * mm + e_u[t];"),
    "error feedback ratio inverted": ("sams_oracle_impl.h", "e_u[t] = mm + rho * e_u[t];", "e_u[t] = mm + e_u[t] / rho;"),
    "h is a sum": ("sams_oracle_impl.h", "h = acc / (REAL)n;", "h = acc;"),
    "v fed on every coordinate": ("sams_oracle_impl.h", "if (in_prev && in_prev[l]) {", "if (1) {"),
    "no max in vhat": ("sams_oracle_impl.h", "if (vv > vhat[l]) vhat[l] = vv;", "vhat[l] = vv;"),
    "v uses h, not h^2": ("sams_oracle_impl.h", "omb2 * (h * h)", "omb2 * h"),
    "e not cleared on the index set": ("sams_oracle_impl.h", "e_u[(int64_t)i * d + l] = (REAL)0;", "(void)e_u;"),
    "x moves the wrong way": ("sams_oracle_impl.h", "x[l] = x[l] - lr * delta[q];", "x[l] = x[l] + lr * delta[q];"),
}

PINS = [  # cheap first; a mutant is caught as soon as one of them fails
    pins.test_hash_matches_bigint_arithmetic_random_and_edges,
    pins.test_hash_dump_matches_bigint,
    pins.test_sketch_mean_adds_workers_in_ascending_order,
    pins.test_gather_and_tail_small_example_by_hand,
    lambda: pins.test_topk_matches_full_sort_with_ties("f64"),
    lambda: pins.test_unsketch_is_rowwise_median_brute_force(2),
    lambda: pins.test_unsketch_is_rowwise_median_brute_force(5),
    pins.test_sketch_linearity_is_bit_exact_on_integer_inputs,
    pins.test_sketch_equals_dense_signed_matrix_product,
    pins.test_single_coordinate_closed_form,
    pins.test_k_equals_d_degenerates_to_distributed_amsgrad,
    pins.test_exact_recovery_equals_dense_topk_error_feedback_amsgrad,
    pins.test_lemma3_auxiliary_sequence_and_structural_invariants,
    pins.test_lemma3_holds_with_a_decaying_step_size,
    lambda: pins.test_refine_matches_full_sort_with_ties("f64"),
    pins.test_pa_single_coordinate_closed_form,
    pins.test_pa_without_compression_averages_per_worker_amsgrad_steps,
    pins.test_pa_auxiliary_sequence_identity_with_decaying_step_size,
    pins.test_sketch_then_unsketch_meets_count_sketch_error_bound,
]


@pytest.mark.parametrize("name", list(MUTANTS))
def test_a_planted_mistake_is_caught(name, tmp_path):
    fname, old, new = MUTANTS[name]
    for f in ("sams_oracle.c", "sams_oracle_impl.h"):
        shutil.copy(os.path.join(HERE, f), tmp_path / f)
    text = (tmp_path / fname).read_text()
    assert text.count(old) >= 1, f"mutation site not found: {old!r}"
    (tmp_path / fname).write_text(text.replace(old, new))
    so = str(tmp_path / "libmutant.so")
    subprocess.check_call(["gcc", *[f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")], "-w",
                           str(tmp_path / "sams_oracle.c"), "-o", so, "-lm"])
    caught = None
    oracle.use_library(so)
    try:
        for pin in PINS:
            try:
                pin()
            except AssertionError:
                caught = getattr(pin, "__name__", "pin")
                break
    finally:
        oracle.use_library(None)
    assert caught is not None, f"no pin noticed: {name}"


def test_the_real_oracle_passes_the_same_pins():
    for pin in PINS:
        pin()
