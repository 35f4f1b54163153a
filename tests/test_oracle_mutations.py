"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C
source (a dropped term, a wrong sign, a wrong index, a flipped tie-break, an unsigned
byte, a forgotten scale, ...), builds it, points the oracle's Python wrapper at the
mutated library and re-runs the pin tests: at least one of them has to fail.  The mistakes
live in the oracle, on the CPU; the product code is not involved."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from oracle import ivf_oracle as O
import tests.test_oracle_int8 as P8
import tests.test_oracle_pins as P

SRC = open(os.path.join(os.path.dirname(O.__file__), "ivf_oracle.c")).read()

MUTATIONS = [
    ("coarse drops the last dimension",
     "for (int t = 0; t < d; ++t)\n                s += (double)Q[q * d + t] * (double)C[j * d + t];",
     "for (int t = 0; t + 1 < d; ++t)\n                s += (double)Q[q * d + t] * (double)C[j * d + t];"),
    ("coarse with the wrong sign",
     "s += (double)Q[q * d + t] * (double)C[j * d + t];", "s -= (double)Q[q * d + t] * (double)C[j * d + t];"),
    ("coarse reads the query of the wrong row",
     "s += (double)Q[q * d + t] * (double)C[j * d + t];", "s += (double)Q[t] * (double)C[j * d + t];"),
    ("scan drops the first dimension",
     "for (int t = 0; t < d; ++t)\n        s += (double)q[t] * elem(X, dtype, i * d + t);",
     "for (int t = 1; t < d; ++t)\n        s += (double)q[t] * elem(X, dtype, i * d + t);"),
    ("scan reads the neighbouring vector",
     "s += (double)q[t] * elem(X, dtype, i * d + t);", "s += (double)q[t] * elem(X, dtype, (i > 0 ? i - 1 : i) * d + t);"),
    ("scan accumulates in single precision",
     "static double stored_dot(const void *X, int dtype, int64_t i, int d, const float *q)\n{\n    double s = 0.0;",
     "static double stored_dot(const void *X, int dtype, int64_t i, int d, const float *q)\n{\n    float s = 0.0;"),
    ("ties on the score go to the larger id",
     "if (x->id < y->id) return -1;\n    if (x->id > y->id) return 1;", "if (x->id < y->id) return 1;\n    if (x->id > y->id) return -1;"),
    ("results come out worst first",
     "if (x->s > y->s) return -1;\n    if (x->s < y->s) return 1;", "if (x->s > y->s) return 1;\n    if (x->s < y->s) return -1;"),
    ("every query uses the probes of query 0",          # in both loops, so the candidate buffer still fits
     "int32_t l = probes[q * nprobe + r];", "int32_t l = probes[r];"),
    ("the last vector of a list is skipped",
     "for (int64_t i = offsets[l]; i < offsets[l + 1]; ++i) {", "for (int64_t i = offsets[l]; i + 1 < offsets[l + 1]; ++i) {"),
    ("padding uses id 0", "out_ids[q * kout + r] = -1;", "out_ids[q * kout + r] = 0;"),
    ("half decoder with the wrong exponent bias", "ldexp(1.0 + (double)f / 1024.0, e - 15)", "ldexp(1.0 + (double)f / 1024.0, e - 14)"),
    ("half decoder ignores subnormals", "v = ldexp((double)f, -24);", "v = 0.0;"),
    ("int8 codes read as unsigned", "(double)(signed char)row[t]", "(double)row[t]"),
    ("int8 scale forgotten", "return (double)scale * s;", "return s;"),
    ("int8 scale read from the wrong place", "memcpy(&scale, row + d, sizeof scale);", "memcpy(&scale, row + d - 4, sizeof scale);"),
    ("assignment breaks ties high", "if (s > bs) { bs = s; bj = j; }", "if (s >= bs) { bs = s; bj = j; }"),
    ("probe selection returns one list twice", "probes[q * nprobe + r] = (int32_t)c[r].id;", "probes[q * nprobe + r] = (int32_t)c[r > 0 ? r - 1 : 0].id;"),
]


def _pin_calls():
    """The pin tests, as callables (parametrised ones with a few of their cases)."""
    calls = [
        P.test_half_decoder_matches_numpy_on_all_bit_patterns,
        lambda: P.test_all_lists_probed_equals_exhaustive_search(0, np.float32, 5),
        lambda: P.test_all_lists_probed_equals_exhaustive_search(1, np.float16, 10),
        lambda: P.test_inner_product_ranking_equals_library_l2_knn_on_unit_vectors(0),
        lambda: P.test_closed_form_basis_case_from_golden_file(np.float32),
        lambda: P.test_closed_form_basis_case_from_golden_file(np.float16),
        P.test_every_returned_score_is_the_dot_product_of_its_vector,
        P.test_prefix_property_and_merge_property_of_selection,
        P.test_monotone_in_nprobe_and_full_recall_at_nlist,
        P.test_probe_ties_go_to_the_smaller_list_and_nprobe_is_clamped,
        P.test_score_ties_go_to_the_smaller_id_then_position,
        P.test_assign_matches_library_argmax_and_breaks_ties_low,
        P.test_rows_do_not_depend_on_batch_or_on_order_inside_a_list_or_on_list_labels,
        lambda: P8.test_all_lists_probed_equals_exhaustive_search_over_dequantised_vectors(1, 5),
        P8.test_every_returned_score_is_scale_times_the_dot_product_with_the_codes,
        P8.test_integer_vectors_with_unit_scale_reduce_to_the_float32_routine,
        P8.test_closed_form_basis_case_survives_quantisation,
    ]
    return calls


def _load(path):
    lib = C.CDLL(path)
    lib.oracle_half_to_double.restype = C.c_double
    lib.oracle_half_to_double.argtypes = [C.c_uint16]
    lib.oracle_threads.restype = C.c_int
    for name in ("oracle_coarse", "oracle_probe_select", "oracle_scan_select", "oracle_assign"):
        getattr(lib, name).restype = C.c_int
    return lib


def _failures():
    n = 0
    for call in _pin_calls():
        try:
            call()
        except AssertionError:
            n += 1
    return n


def test_unmutated_oracle_passes_every_pin_used_here():
    O.lib()
    assert _failures() == 0


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_is_caught(name, old, new, tmp_path):
    assert SRC.count(old) >= 1, f"mutation '{name}' no longer matches the oracle source"
    src = tmp_path / "mutant.c"
    src.write_text(SRC.replace(old, new))          # every occurrence: a mutant must stay memory-safe
    so = str(tmp_path / "mutant.so")
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", so, str(src), "-lm"])
    good = O.lib()
    try:
        O._lib = _load(so)
        caught = _failures()
    finally:
        O._lib = good
    assert caught >= 1, f"no pin notices: {name}"


# ------------------------------------------------------------ the batch-scheduling oracle
import importlib.util
import types

import tests.test_batch_sched as PB
from oracle import batch_sched_oracle as SO

SO_SRC = open(SO.__file__).read()

SCHED_MUTATIONS = [
    ("Eq. 6 with k/2 instead of (k+1)/2", "return (k + 1) / 2.0 * batch_time(a, c, n / k) - mean_arrival", "return k / 2.0 * batch_time(a, c, n / k) - mean_arrival"),
    ("Eq. 6 with batches of n instead of n/k", "batch_time(a, c, n / k) - mean_arrival", "batch_time(a, c, n) - mean_arrival"),
    ("mean arrival time added instead of subtracted", "batch_time(a, c, n / k) - mean_arrival", "batch_time(a, c, n / k) + mean_arrival"),
    ("Eq. 4 with the exponent on a", "return a * B ** c", "return (a * B) ** c"),
    ("Eq. 7 with k^c instead of 2 k^c", "return 2.0 * k ** c <= k + 1", "return k ** c <= k + 1"),
    ("Eq. 7 with k instead of k+1", "return 2.0 * k ** c <= k + 1", "return 2.0 * k ** c <= k"),
    ("threshold with the wrong logarithm", "return math.log((k + 1) / 2.0) / math.log(k)", "return math.log((k + 1) / 2.0) / math.log(2 * k)"),
    ("fit returns the slope of T on B", "ys = [math.log(t) for t in Ts]", "ys = [t for t in Ts]"),
    ("the last, smaller batch is charged T(B)", "total += r * (m * tB + batch_time(a, c, r))", "total += r * (m * tB + tB)"),
    ("the last batch does not wait for the full ones", "total += r * (m * tB + batch_time(a, c, r))", "total += r * batch_time(a, c, r)"),
    ("full batches counted m(m-1)/2 times", "total = B * tB * m * (m + 1) / 2.0", "total = B * tB * m * (m - 1) / 2.0"),
    ("average over the full batches only", "return total / n - mean_arrival", "return total / max(1, m * B) - mean_arrival"),
    ("ties go to the smaller batch", "(L == best_L and B > best_B)", "(L == best_L and B < best_B)"),
    ("the worst candidate wins", "L < best_L or", "L > best_L or"),
]


def _sched_pins():
    calls = []
    for a, c in [(0.7, 0.0), (1.3, 0.3), (0.5, 1.7)]:
        for n, k in [(64, 1), (64, 4), (60, 3)]:
            calls.append(lambda a=a, c=c, n=n, k=k: PB.test_equations_5_and_6_equal_a_simulation_of_serial_batches(a, c, n, k))
    calls += [lambda k=k: PB.test_equation_7_is_the_comparison_of_equations_5_and_6(k) for k in (2, 4, 16)]
    calls += [PB.test_k2_threshold_is_the_value_the_paper_prints,
              PB.test_fit_recovers_an_exact_power_law_and_matches_a_library_polyfit,
              PB.test_choice_follows_the_scaling_exponent,
              PB.test_choice_with_a_queue_no_candidate_divides_is_the_simulated_best]
    for n, B in [(20, 8), (20, 32), (7, 3), (64, 16)]:
        calls.append(lambda n=n, B=B: PB.test_a_batch_size_that_does_not_divide_the_queue_equals_the_simulation(1.3, 0.3, n, B))
    return calls


def _sched_failures():
    n = 0
    for call in _sched_pins():
        try:
            call()
        except AssertionError:
            n += 1
    return n


def test_unmutated_scheduling_oracle_passes_its_pins():
    assert _sched_failures() == 0


@pytest.mark.parametrize("name,old,new", SCHED_MUTATIONS, ids=[m[0] for m in SCHED_MUTATIONS])
def test_a_planted_mistake_in_the_scheduling_oracle_is_caught(name, old, new):
    assert SO_SRC.count(old) >= 1, f"mutation '{name}' no longer matches the oracle source"
    mutant = types.ModuleType("mutant_batch_sched_oracle")
    exec(compile(SO_SRC.replace(old, new), "mutant_batch_sched_oracle.py", "exec"), mutant.__dict__)
    good = PB.SO
    try:
        PB.SO = mutant
        caught = _sched_failures()
    finally:
        PB.SO = good
    assert caught >= 1, f"no pin notices: {name}"


# ------------------------------------------------------------ the product-quantisation oracle
import tests.test_oracle_pq as PP
from oracle import pq_oracle as PQO

PQ_SRC = open(PQO.__file__).read().replace("from . import ivf_oracle as O", "from oracle import ivf_oracle as O")

PQ_MUTATIONS = [
    ("subspace slices overlap", "qm = q[m * dsub:(m + 1) * dsub].astype(np.float64)", "qm = q[m:m + dsub].astype(np.float64)"),
    ("codebook of the wrong subspace", "T[m] += qm[t] * codebooks[m][:, t].astype(np.float64)", "T[m] += qm[t] * codebooks[0][:, t].astype(np.float64)"),
    ("a dimension of every subspace dropped", "for t in range(dsub):", "for t in range(dsub - 1):"),
    ("last subspace left out of the score", "for m in range(T.shape[0]):", "for m in range(T.shape[0] - 1):"),
    ("codes read transposed", "s += T[m][codes[:, m]]", "s += T[m][codes[:, T.shape[0] - 1 - m]]"),
    ("table entries subtracted", "s += T[m][codes[:, m]]", "s -= T[m][codes[:, m]]"),
    ("worst candidates first", "order = np.lexsort((pos, ids[pos], -s))[:kout]", "order = np.lexsort((pos, ids[pos], s))[:kout]"),
    ("ties to the larger id", "order = np.lexsort((pos, ids[pos], -s))[:kout]", "order = np.lexsort((pos, -ids[pos], -s))[:kout]"),
    ("decode copies the wrong codeword", "out[:, m * dsub:(m + 1) * dsub] = codebooks[m][codes[:, m]]", "out[:, m * dsub:(m + 1) * dsub] = codebooks[m][255 - codes[:, m]]"),
    ("one probed list skipped", "for l in probes[r]]", "for l in probes[r][1:]]"),
]


def _pq_pins():
    calls = [PP.test_hand_worked_case,
             PP.test_codes_that_reproduce_their_vectors_reduce_to_the_flat_search_on_the_originals]
    calls += [lambda s=s: PP.test_table_scores_equal_a_library_matmul_against_the_decoded_vectors(s) for s in (0, 1)]
    calls += [lambda k=k: PP.test_all_lists_probed_equals_exhaustive_search_over_the_decoded_vectors(0, k) for k in (1, 10, 600)]
    calls += [lambda: PP.test_matches_the_flat_oracle_on_the_decoded_vectors_for_any_nprobe(0)]
    return calls


def _pq_failures():
    n = 0
    for call in _pq_pins():
        try:
            call()
        except AssertionError:
            n += 1
    return n


def test_unmutated_pq_oracle_passes_its_pins():
    assert _pq_failures() == 0


@pytest.mark.parametrize("name,old,new", PQ_MUTATIONS, ids=[m[0] for m in PQ_MUTATIONS])
def test_a_planted_mistake_in_the_pq_oracle_is_caught(name, old, new):
    assert PQ_SRC.count(old) >= 1, f"mutation '{name}' no longer matches the oracle source"
    mutant = types.ModuleType("mutant_pq_oracle")
    exec(compile(PQ_SRC.replace(old, new), "mutant_pq_oracle.py", "exec"), mutant.__dict__)
    good = PP.PQ
    try:
        PP.PQ = mutant
        caught = _pq_failures()
    finally:
        PP.PQ = good
    assert caught >= 1, f"no pin notices: {name}"
