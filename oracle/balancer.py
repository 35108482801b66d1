"""CPU oracle for the workload model, the compute-bag topology string and the
greedy balancer.

TEST INFRASTRUCTURE ONLY: imported by the tests (and the smoke check), never by
the library, and sharing no code with the C implementation in the library.

The greedy balancer is a heuristic, so its oracle is the algorithm itself,
taken step by step in the order of Sec. 3.3 (first and second pass) with the
workload model of Sec. 3.1 (Eq. 1 and Eq. 2), the topology string of Sec. 3.2
and the workload-imbalance ratio defined in Sec. 4.2.  Readings where the text
is silent (marked READING below):

* no bag has enough remaining capacity: the text does not say; it must happen,
  because capacities sum exactly to the total load and a single sequence can
  outweigh a whole bag.  READING: then every bag is a candidate.
* ties: READING: stable descending order of workload (original index breaks
  ties); the lowest bag index wins among equal occupancies.
* "sufficient" means remaining capacity >= w_i in exact float64 comparison.
* a sequence put into a g-GPU bag adds its whole w_i to that bag; each GPU of
  the bag then carries load/g (Sec. 3.4: equal heads per worker make the split
  of attention work equal).
* uneven chunks in the second pass: READING: the first (L mod g) chunks get
  one more token.

Pins (tests/test_oracle_balancer.py): exhaustive optimum on tiny instances with
the LPT bound for equal bags, conservation invariants, and the WIR cells the
paper prints in Table 1.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def flux_workload(l: float, d_model: float, gamma: float = 1.0) -> float:
    """Eq. 2 without the hardware constant k: 24 l d^2 + gamma 4 l^2 d (Eq. 1 when gamma = 1)."""
    return 24.0 * l * d_model * d_model + gamma * 4.0 * l * l * d_model


def seq_cost(L: float, a: float, b: float) -> float:
    """The same model in the form a L^2 + b L (a = k gamma 4 d, b = k 24 d^2)."""
    return a * L * L + b * L


def gamma_equivalent(a: float, b: float, d_model: float) -> float:
    """gamma such that a L^2 + b L is proportional to Eq. 2: gamma = 6 d a / b."""
    return 6.0 * d_model * a / b


def parse_topology(spec: str) -> List[int]:
    """'g1n2+g2n1+g4n1' -> [1, 1, 2, 4]: each term g{G}n{N} is N bags of G GPUs (Sec. 3.2)."""
    bags: List[int] = []
    for term in spec.strip().split("+"):
        term = term.strip()
        if not term.startswith("g") or "n" not in term:
            raise ValueError(f"bad topology term {term!r}")
        g_str, n_str = term[1:].split("n", 1)
        g, n = int(g_str), int(n_str)
        if g <= 0 or n <= 0:
            raise ValueError(f"bad topology term {term!r}")
        bags.extend([g] * n)
    return bags


def greedy_assign(weights: Sequence[float], bag_gpus: Sequence[int]) -> Tuple[List[int], List[float]]:
    """First pass of Sec. 3.3.  Returns (bag index of every sequence, load of every bag)."""
    w = [float(x) for x in weights]
    G = int(sum(bag_gpus))
    target = sum(w) / G                                   # per-GPU target workload
    cap = [g * target for g in bag_gpus]                  # bag capacity
    load = [0.0] * len(bag_gpus)
    bag_of = [-1] * len(w)
    order = sorted(range(len(w)), key=lambda i: (-w[i], i))   # descending, stable
    for i in order:
        fits = [j for j in range(len(cap)) if cap[j] - load[j] >= w[i]]
        cand = fits if fits else list(range(len(cap)))    # READING: fall back to all bags
        best = cand[0]
        for j in cand[1:]:
            if load[j] / cap[j] < load[best] / cap[best]:  # lowest occupancy, lowest index on ties
                best = j
        load[best] += w[i]
        bag_of[i] = best
    return bag_of, load


def chunk_lengths(L: int, g: int) -> List[int]:
    """Second pass of Sec. 3.3: g contiguous chunks, as even as possible."""
    base, rem = divmod(int(L), int(g))
    return [base + (1 if c < rem else 0) for c in range(g)]


def wir(bag_load: Sequence[float], bag_gpus: Sequence[int]) -> float:
    """Workload imbalance ratio: max over min of the per-GPU workloads (Sec. 4.2)."""
    per_gpu = [l / g for l, g in zip(bag_load, bag_gpus)]
    lo = min(per_gpu)
    return float("inf") if lo <= 0.0 else max(per_gpu) / lo


def bag_sequences(seq_lens: Sequence[int], bag_of: Sequence[int], bag: int) -> List[int]:
    """The sequences of one bag in their original order (that bag's packed list)."""
    return [int(l) for l, b in zip(seq_lens, bag_of) if b == bag]


def fit_cost_model(sum_l2: Sequence[float], sum_l: Sequence[float], t: Sequence[float]):
    """Least squares of t ~ a*sumL2 + b*sumL on relative error (weights 1/t^2), no intercept.

    Sec. 3.1 obtains the correction factor by fitting the model to measured
    (l, t) pairs; the objective is not stated.  READING: relative least squares.
    Returns (a, b, max relative residual).
    """
    x2 = np.asarray(sum_l2, dtype=np.float64)
    x1 = np.asarray(sum_l, dtype=np.float64)
    tt = np.asarray(t, dtype=np.float64)
    A = np.stack([x2 / tt, x1 / tt], axis=1)        # rows scaled by 1/t -> relative residuals
    rhs = np.ones_like(tt)
    (a, b), *_ = np.linalg.lstsq(A, rhs, rcond=None)
    resid = np.abs(a * x2 + b * x1 - tt) / tt
    return float(a), float(b), float(resid.max())
