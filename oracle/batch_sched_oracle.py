"""CPU oracle for the backlog-aware batch-size choice of the retrieval worker.
TEST INFRASTRUCTURE ONLY (tests and the benchmark's reporting); shares no code with the
library's implementation.

Follows Section 4.4, "Backlog-aware Batch Scheduling (Online)", in the paper's order and
notation, in plain fp64 Python:

  T(B)  = a * B**c, a > 0, c >= 0                      processing time of a batch of B   (Eq. 4)
  L_1   = T(n) - mean(t_i)                             one batch with all n requests     (Eq. 5)
  L_k   = (k+1)/2 * T(n/k) - mean(t_i)                 k equal batches, served in turn   (Eq. 6)
  one batch is at least as good as k batches  <=>  2 * k**c <= k + 1                     (Eq. 7)
  for k = 2:  c <= log2(3/2) ~ 0.585                                                     (Eq. 8)

"In practice" (same section): with n requests queued, the candidate batch sizes (the
paper's example: 8, 16, 32, 64 for n = 64) are scored with these formulas using T from
profiled samples, and the best one is taken.

Readings where the text is silent: (a, c) are fitted to profiled (B, T) samples by least
squares on log T = log a + c log B; a candidate B that does not divide n (the equations
only cover equal batches) is scored by the same derivation as Eq. 6 applied to what the
worker would actually serve: m = floor(n/B) batches of B, then one batch of the
r = n - m*B requests that are left, which takes T(r).  A request's latency is the
completion time of its batch minus its arrival, so
L(B) = [ B * T(B) * m(m+1)/2 + r * (m * T(B) + T(r)) ] / n - mean(t_i),
which is Eq. 6 for r = 0 and Eq. 5 for B >= n (m = 0, r = n); ties go to the larger batch
(fewer launches).

Pins (tests/test_batch_sched.py): an event-by-event simulation of serving the batches
one after the other, request by request, reproduces Eq. 5/6 and the unequal-last-batch
formula; Eq. 7 agrees with comparing Eq. 5 and Eq. 6 directly; the k = 2 threshold is the
value the paper prints (tests/golden/).
"""
from __future__ import annotations

import math
from typing import Iterable, Sequence, Tuple


def batch_time(a: float, c: float, B: float) -> float:
    return a * B ** c


def fit_power_law(Bs: Sequence[float], Ts: Sequence[float]) -> Tuple[float, float]:
    xs = [math.log(b) for b in Bs]
    ys = [math.log(t) for t in Ts]
    m = len(xs)
    mx, my = sum(xs) / m, sum(ys) / m
    sxx = sum((x - mx) ** 2 for x in xs)
    if sxx == 0.0:
        return math.exp(my), 0.0
    c = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sxx
    return math.exp(my - c * mx), c


def avg_latency_equal_batches(a: float, c: float, n: int, k: int, mean_arrival: float = 0.0) -> float:
    """Eq. 5 (k = 1) and Eq. 6."""
    return (k + 1) / 2.0 * batch_time(a, c, n / k) - mean_arrival


def single_batch_is_best(c: float, k: int) -> bool:
    """Eq. 7."""
    return 2.0 * k ** c <= k + 1


def split_threshold(k: int) -> float:
    """Largest c for which one batch is still at least as good as k batches (Eq. 7 solved
    for c); k = 2 gives Eq. 8."""
    return math.log((k + 1) / 2.0) / math.log(k)


def candidate_latency(a: float, c: float, n: int, B: int, mean_arrival: float = 0.0) -> float:
    m = n // B                           # full batches of B (none if B > n)
    r = n - m * B                        # requests left for the last, smaller batch
    tB = batch_time(a, c, B)
    total = B * tB * m * (m + 1) / 2.0
    if r > 0:
        total += r * (m * tB + batch_time(a, c, r))
    return total / n - mean_arrival


def choose_batch_size(a: float, c: float, n: int, candidates: Iterable[int],
                      mean_arrival: float = 0.0) -> Tuple[int, float]:
    best_B, best_L = None, None
    for B in candidates:
        L = candidate_latency(a, c, n, B, mean_arrival)
        if best_L is None or L < best_L or (L == best_L and B > best_B):
            best_B, best_L = B, L
    return best_B, best_L
