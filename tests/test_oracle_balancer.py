"""Pins of the balancer / workload-model oracle.

* the WIR cells the paper prints in Table 1 (tests/golden/table1_wir.txt);
* the token counts and HFU cells of Table 1, which fix the data-code token
  rule and Eq. 1 as the FLOP count (tests/golden/table1_throughput.txt);
* exhaustive optimum on tiny instances with the LPT bound (equal bags make the
  rule longest-processing-time list scheduling);
* conservation invariants; the topology string example of Sec. 3.2.
"""
import itertools
import os

import numpy as np
import pytest

from knap_inputs import table1_streams
from oracle import balancer as B

GOLD = os.path.join(os.path.dirname(__file__), "golden")
D_MODEL, GAMMA = 3072, 0.49       # Table 1 caption


def _read(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _wir_for(workload, topo, seed=None):
    per_gpu = table1_streams(workload, seed)
    if topo == "none":
        loads = [sum(B.flux_workload(l, D_MODEL, GAMMA) for l in g) for g in per_gpu]
        return max(loads) / min(loads)
    lens = [l for g in per_gpu for l in g]
    w = [B.flux_workload(l, D_MODEL, GAMMA) for l in lens]
    bags = B.parse_topology(topo)
    _, load = B.greedy_assign(w, bags)
    return B.wir(load, bags)


def test_topology_string_example():
    assert B.parse_topology("g1n2+g2n1+g4n1") == [1, 1, 2, 4]
    assert B.parse_topology("g8n4") == [8, 8, 8, 8]
    with pytest.raises(ValueError):
        B.parse_topology("g0n1")
    with pytest.raises(ValueError):
        B.parse_topology("x1n1")


def test_table1_wir_cells_mean_streams():
    """Deterministic mean-length streams (196 text tokens, no aspect jitter).

    Balanced cells of the paper are reproduced to +-0.03 (g2n16, g4n8, g8n4)
    and +-0.2 (g1n32: one sequence outweighs a whole bag there, so the cell
    is sensitive to the random text lengths the paper drew).
    """
    for workload, topo, val in _read("table1_wir.txt"):
        val = float(val)
        if topo == "none":
            continue
        got = _wir_for(workload, topo)
        tol = 0.2 if topo == "g1n32" else 0.03
        assert abs(got - val) <= tol, (workload, topo, got, val)


def test_table1_wir_cells_mean_streams_to_three_decimals():
    """The mean-length streams are deterministic, and so is the greedy pass with its tie-breaks (stable
    descending sort, lowest bag index among equal occupancies, every bag a candidate when none has room):
    its eight balanced cells of the mixed_res and joint workloads, taken from an evaluation of
    Sec. 3.3's steps on those streams made independently of this oracle, are fixed here to three decimals, inside the bands around the printed cells above.
    A changed tie-break moves the third decimal long before it leaves a band."""
    want = {("mixed_res", "g1n32"): 3.882, ("mixed_res", "g2n16"): 1.276, ("mixed_res", "g4n8"): 1.002,
            ("mixed_res", "g8n4"): 1.000, ("joint", "g1n32"): 4.766, ("joint", "g2n16"): 1.640,
            ("joint", "g4n8"): 1.006, ("joint", "g8n4"): 1.002}
    for (workload, topo), val in want.items():
        assert abs(_wir_for(workload, topo) - val) < 5e-4, (workload, topo, _wir_for(workload, topo), val)
    for topo in ("g1n32", "g2n16", "g4n8", "g8n4"):
        assert abs(_wir_for("low_res", topo) - 1.0) < 5e-4


def test_table1_wir_cells_random_streams():
    """With random text lengths and aspect jitter the cells stay in the same bands,
    and the unbalanced ratio lands in the paper's order of magnitude."""
    printed = {(w, t): float(v) for w, t, v in _read("table1_wir.txt")}
    for workload in ("low_res", "mixed_res", "joint"):
        for topo in ("g1n32", "g2n16", "g4n8", "g8n4"):
            vals = [_wir_for(workload, topo, seed) for seed in range(5)]
            tol = 0.6 if topo == "g1n32" else 0.12
            assert abs(float(np.median(vals)) - printed[(workload, topo)]) <= tol, (workload, topo, vals)
        unb = [_wir_for(workload, "none", seed) for seed in range(5)]
        ref = printed[(workload, "none")]
        assert 0.5 * ref <= float(np.median(unb)) <= 1.6 * ref, (workload, unb)


def test_table1_token_counts_and_hfu_fix_eq1():
    """TPS x FBL = tokens per step from the data codes, and HFU follows from
    4 x 57 blocks x (24 d^2 + 4 d sum(l^2)/sum(l)) per token at one common peak."""
    peaks = []
    for workload, topo, fbl, tps_k, hfu in _read("table1_throughput.txt"):
        fbl, tps, hfu = float(fbl), float(tps_k) * 1e3, float(hfu) / 100.0
        lens = [l for g in table1_streams(workload) for l in g]
        tokens = sum(lens)
        assert abs(tps * fbl - tokens) / tokens <= 0.005, (workload, topo, tps * fbl, tokens)
        fwd_flops_step = 57 * sum(B.flux_workload(l, D_MODEL, 1.0) for l in lens)
        peaks.append(4.0 * fwd_flops_step / fbl / 32.0 / hfu)
    peaks = np.array(peaks)
    # every cell implies the same per-GPU peak (~989 TFLOP/s, H100 dense bf16)
    assert np.all(np.abs(peaks / 989e12 - 1.0) <= 0.01), peaks


def _exhaustive_best_makespan(w, m):
    best = float("inf")
    for assign in itertools.product(range(m), repeat=len(w)):
        loads = [0.0] * m
        for wi, j in zip(w, assign):
            loads[j] += wi
        best = min(best, max(loads))
    return best


def test_equal_bags_is_lpt_and_within_its_bound():
    rng = np.random.default_rng(0)
    for trial in range(30):
        n = int(rng.integers(3, 9))
        m = int(rng.integers(2, 4))
        w = [float(x) for x in rng.uniform(1.0, 10.0, size=n)]
        bag_of, load = B.greedy_assign(w, [1] * m)
        # plain LPT: sort descending, always the least-loaded machine
        lpt = [0.0] * m
        for wi in sorted(w, reverse=True):
            lpt[int(np.argmin(lpt))] += wi
        assert sorted(load) == pytest.approx(sorted(lpt), rel=0, abs=1e-12)
        opt = _exhaustive_best_makespan(w, m)
        assert max(load) <= (4.0 / 3.0 - 1.0 / (3.0 * m)) * opt + 1e-9
        assert max(load) >= opt - 1e-9


def test_conservation_and_determinism():
    rng = np.random.default_rng(1)
    lens = [int(x) for x in rng.integers(100, 30000, size=200)]
    w = [B.seq_cost(l, 2.0e-9, 3.0e-6) for l in lens]
    bags = B.parse_topology("g1n2+g2n1+g4n1")
    bag_of, load = B.greedy_assign(w, bags)
    assert all(0 <= b < len(bags) for b in bag_of)
    assert sum(load) == pytest.approx(sum(w), rel=1e-12)
    for j in range(len(bags)):
        assert load[j] == pytest.approx(sum(wi for wi, b in zip(w, bag_of) if b == j), rel=1e-12)
    assert (bag_of, load) == B.greedy_assign(w, bags)
    # bigger bags receive proportionally more work: per-GPU loads are close
    assert B.wir(load, bags) < 1.01
    assert sum(len(B.bag_sequences(lens, bag_of, j)) for j in range(len(bags))) == len(lens)


def test_oversized_sequence_falls_back_to_lowest_occupancy():
    # one item heavier than any capacity: every bag is a candidate, lowest occupancy wins
    w = [100.0, 1.0, 1.0, 1.0]
    bag_of, load = B.greedy_assign(w, [1, 1])
    assert bag_of[0] == 0 and bag_of[1:] == [1, 1, 1]
    assert load == [100.0, 3.0]


def test_capacity_filter_prefers_a_bag_where_the_sequence_fits():
    # target per GPU = 10, capacities [10, 30].  After 9 -> bag 0 (both empty, index 0)
    # and 8 -> bag 1, the 6 does not fit in bag 0 (1 left) although ... occupancy check:
    w = [9.0, 8.0, 6.0, 6.0, 6.0, 5.0]
    bags = [1, 3]
    bag_of, load = B.greedy_assign(w, bags)
    assert bag_of == [0, 1, 1, 1, 1, 1]
    assert load == [9.0, 31.0]


def test_chunks_and_model_forms():
    assert B.chunk_lengths(10, 4) == [3, 3, 2, 2]
    assert B.chunk_lengths(8, 8) == [1] * 8
    assert sum(B.chunk_lengths(16580, 8)) == 16580
    # Eq. 1 and Eq. 2
    assert B.flux_workload(10, 4, 1.0) == 24 * 10 * 16 + 4 * 100 * 4
    assert B.flux_workload(10, 4, 0.5) == 24 * 10 * 16 + 0.5 * 4 * 100 * 4
    # a L^2 + b L with a = k gamma 4 d, b = k 24 d^2 is k x Eq. 2, and gamma is recovered
    kk, gamma, d = 1e-12, 0.385, 3072
    a, b = kk * gamma * 4 * d, kk * 24 * d * d
    assert B.seq_cost(5000, a, b) == pytest.approx(kk * B.flux_workload(5000, d, gamma), rel=1e-14)
    assert B.gamma_equivalent(a, b, d) == pytest.approx(gamma, rel=1e-14)


def test_fit_recovers_known_constants():
    rng = np.random.default_rng(2)
    a, b = 3.1e-9, 4.2e-6
    L = np.array([256, 512, 1024, 2048, 4096, 8192, 16384, 32768, 65536], dtype=np.float64)
    t = a * L * L + b * L
    a2, b2, r = B.fit_cost_model(L * L, L, t)
    assert a2 == pytest.approx(a, rel=1e-10) and b2 == pytest.approx(b, rel=1e-10) and r < 1e-10
    noisy = t * (1.0 + 0.01 * rng.standard_normal(t.shape))
    a3, b3, r3 = B.fit_cost_model(L * L, L, noisy)
    assert a3 == pytest.approx(a, rel=0.05) and b3 == pytest.approx(b, rel=0.05) and r3 < 0.05


def test_bag_sequences_hand_case_keeps_original_order():
    # six sequences dealt to three bags by hand: a bag's packed list is its members in the order they
    # arrived, duplicates of a length stay apart, an unused bag is empty
    lens = [5, 3, 8, 3, 1, 7]
    bag_of = [1, 0, 1, 1, 0, 1]
    assert B.bag_sequences(lens, bag_of, 0) == [3, 1]
    assert B.bag_sequences(lens, bag_of, 1) == [5, 8, 3, 7]
    assert B.bag_sequences(lens, bag_of, 2) == []
    # the bags partition the multiset of lengths
    assert sorted(B.bag_sequences(lens, bag_of, 0) + B.bag_sequences(lens, bag_of, 1)) == sorted(lens)
