"""Backlog-aware batch-size choice (paper Section 4.4, Eq. 4-8): pins for the oracle and
parity of the library's ivf_sched_* functions against it (host arithmetic, no GPU)."""
import math
import os

import numpy as np
import pytest

from oracle import batch_sched_oracle as SO
from paper_2504_15302_amd import ivf

HERE = os.path.dirname(os.path.abspath(__file__))


def _simulate_sizes(a, c, sizes, arrivals):
    """Event-by-event: all requests are queued at time 0 of the clock that the arrival
    times are measured on, batches of the given sizes are served one after the other
    (a batch of s requests takes a * s**c), a request's latency is its batch's completion
    time minus its own arrival time."""
    n = sum(sizes)
    now, lat, i = 0.0, [], 0
    for s in sizes:
        now += a * s ** c                         # this batch finishes
        for _ in range(s):
            lat.append(now - arrivals[i])
            i += 1
    assert i == n == len(arrivals)
    return sum(lat) / n


def _simulate(a, c, n, k, arrivals):
    """k equal batches of n/k."""
    return _simulate_sizes(a, c, [n // k] * k, arrivals)


def _greedy_sizes(n, B):
    """What a worker serves from a queue of n with batch size B: full batches, then the rest."""
    return [B] * (n // B) + ([n % B] if n % B else []) if B < n else [n]


# ------------------------------------------------------------------ oracle pins
@pytest.mark.parametrize("a,c", [(0.7, 0.0), (1.3, 0.3), (0.02, 0.585), (2.0, 1.0), (0.5, 1.7)])
@pytest.mark.parametrize("n,k", [(64, 1), (64, 2), (64, 4), (64, 8), (60, 3), (7, 7)])
def test_equations_5_and_6_equal_a_simulation_of_serial_batches(a, c, n, k):
    rng = np.random.default_rng(n * 31 + k)
    arrivals = (-rng.random(n) * 5.0).tolist()    # requests arrived before the batch was formed
    want = _simulate(a, c, n, k, arrivals)
    got = SO.avg_latency_equal_batches(a, c, n, k, sum(arrivals) / n)
    assert abs(got - want) <= 1e-12 * max(1.0, abs(want))


@pytest.mark.parametrize("k", [2, 3, 4, 8, 16])
def test_equation_7_is_the_comparison_of_equations_5_and_6(k):
    for c in np.linspace(0.0, 1.5, 61):
        l1 = SO.avg_latency_equal_batches(1.0, c, 64 * k, 1)
        lk = SO.avg_latency_equal_batches(1.0, c, 64 * k, k)
        if abs(l1 - lk) > 1e-9 * l1:
            assert SO.single_batch_is_best(c, k) == (l1 <= lk)
    thr = SO.split_threshold(k)
    assert SO.single_batch_is_best(thr - 1e-9, k) and not SO.single_batch_is_best(thr + 1e-9, k)


def test_k2_threshold_is_the_value_the_paper_prints():
    vals = {}
    for line in open(os.path.join(HERE, "golden", "batch_sched_threshold.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            vals[t[0]] = float(t[1])
    thr = SO.split_threshold(int(vals["k"]))
    assert round(thr, int(vals["printed_digits"])) == vals["c_threshold_printed"]
    assert abs(thr - math.log2(1.5)) < 1e-15
    assert SO.single_batch_is_best(0.58, 2) and not SO.single_batch_is_best(0.59, 2)


def test_fit_recovers_an_exact_power_law_and_matches_a_library_polyfit():
    Bs = [8, 16, 32, 64, 128]
    a, c = SO.fit_power_law(Bs, [0.37 * b ** 0.42 for b in Bs])
    assert abs(a - 0.37) < 1e-12 and abs(c - 0.42) < 1e-12
    rng = np.random.default_rng(0)
    Ts = [0.37 * b ** 0.42 * math.exp(rng.normal(0, 0.05)) for b in Bs]
    a, c = SO.fit_power_law(Bs, Ts)
    slope, icpt = np.polyfit(np.log(Bs), np.log(Ts), 1)
    assert abs(c - slope) < 1e-12 and abs(a - math.exp(icpt)) < 1e-12


def test_choice_follows_the_scaling_exponent():
    cands = [8, 16, 32, 64]
    assert SO.choose_batch_size(1.0, 0.1, 64, cands)[0] == 64          # flat time: one big batch
    assert SO.choose_batch_size(1.0, 0.58, 64, cands)[0] == 64
    assert SO.choose_batch_size(1.0, 1.0, 64, cands)[0] == 8           # linear time: smallest batches
    # brute force over the candidates with the simulation
    for c in (0.2, 0.6, 0.8, 1.2):
        sims = {B: _simulate(1.0, c, 64, 64 // B, [0.0] * 64) for B in cands}
        best = min(sims, key=lambda B: (sims[B], -B))
        assert SO.choose_batch_size(1.0, c, 64, cands)[0] == best
    assert SO.choose_batch_size(1.0, 0.3, 20, [32, 64])[0] == 64                # both are one batch of 20: tie -> larger


@pytest.mark.parametrize("a,c", [(0.7, 0.0), (1.3, 0.3), (0.02, 0.585), (2.0, 1.0), (0.5, 1.7)])
@pytest.mark.parametrize("n,B", [(20, 8), (20, 16), (20, 32), (64, 24), (7, 2), (7, 3), (100, 33), (5, 5), (6, 1), (64, 16)])
def test_a_batch_size_that_does_not_divide_the_queue_equals_the_simulation(a, c, n, B):
    """Full batches of B, then the r requests that are left in a batch that takes T(r)."""
    rng = np.random.default_rng(n * 131 + B)
    arrivals = (-rng.random(n) * 3.0).tolist()
    want = _simulate_sizes(a, c, _greedy_sizes(n, B), arrivals)
    got = SO.candidate_latency(a, c, n, B, sum(arrivals) / n)
    assert abs(got - want) <= 1e-12 * max(1.0, abs(want))
    if n % B == 0 and B < n:                      # reduces to Eq. 6
        assert abs(got - SO.avg_latency_equal_batches(a, c, n, n // B, sum(arrivals) / n)) <= 1e-12 * max(1.0, abs(want))


def test_choice_with_a_queue_no_candidate_divides_is_the_simulated_best():
    for c in (0.1, 0.5, 0.7, 1.0, 1.4):
        for n in (20, 37, 50, 63):
            cands = [8, 16, 32, 64]
            sims = {B: _simulate_sizes(1.0, c, _greedy_sizes(n, B), [0.0] * n) for B in cands}
            best_B = min(sims, key=lambda B: (sims[B], -B))
            got_B, got_L = SO.choose_batch_size(1.0, c, n, cands)
            assert abs(got_L - sims[best_B]) <= 1e-12 * sims[best_B]
            # ties (32 and 64 both serve n <= 32 as one batch) go to the larger candidate
            assert got_B == max(B for B in cands if abs(sims[B] - sims[best_B]) <= 1e-15 * sims[best_B])
    assert SO.choose_batch_size(1.0, 0.3, 20, [8, 16, 32, 64])[0] == 64           # flat time: one batch of 20
    assert SO.choose_batch_size(1.0, 1.0, 20, [8, 16, 32, 64])[0] == 8            # linear time: 8 + 8 + 4


# ------------------------------------------------------------------ library vs oracle
def test_library_matches_oracle():
    rng = np.random.default_rng(5)
    for _ in range(200):
        a = float(rng.uniform(0.01, 5.0))
        c = float(rng.uniform(0.0, 1.6))
        n = int(rng.integers(1, 500))
        k = int(rng.integers(1, 20))
        t = float(rng.uniform(-3, 0))
        want = SO.avg_latency_equal_batches(a, c, n, k, t)
        got = ivf.sched_avg_latency(a, c, n, k, t)
        assert abs(got - want) <= 1e-12 * max(1.0, abs(want))
        assert ivf.sched_single_batch_is_best(c, k) == SO.single_batch_is_best(c, k)
        B = float(rng.uniform(1, 300))
        assert abs(ivf.sched_batch_time(a, c, B) - SO.batch_time(a, c, B)) <= 1e-12 * SO.batch_time(a, c, B)
        cands = sorted(set(int(x) for x in rng.integers(1, 200, size=int(rng.integers(1, 6)))))
        gb, gl = ivf.sched_choose(a, c, n, cands, t)
        wb, wl = SO.choose_batch_size(a, c, n, cands, t)
        assert gb == wb and abs(gl - wl) <= 1e-12 * max(1.0, abs(wl))
        m = int(rng.integers(1, 7))
        Bs = rng.choice(np.arange(1, 300), size=m, replace=False).astype(float).tolist()
        Ts = [a * b ** c * math.exp(rng.normal(0, 0.1)) for b in Bs]
        ga, gc = ivf.sched_fit(Bs, Ts)
        wa, wc = SO.fit_power_law(Bs, Ts)
        assert abs(ga - wa) <= 1e-9 * wa and abs(gc - wc) <= 1e-9 * max(1.0, abs(wc))


def test_library_rejects_bad_arguments():
    with pytest.raises(ivf.IvfError):
        ivf.sched_fit([8, -1], [1.0, 2.0])
    with pytest.raises(ivf.IvfError):
        ivf.sched_avg_latency(1.0, 0.5, 0, 1)
    with pytest.raises(ivf.IvfError):
        ivf.sched_choose(1.0, 0.5, 10, [0])
    with pytest.raises(ivf.IvfError):
        ivf.sched_choose(-1.0, 0.5, 10, [4])
