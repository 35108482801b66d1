"""CPU tests of the shared library: it loads, exports every symbol the header
declares, validates arguments, and its host-side model / balancer (C) agrees
with the step-by-step oracle (Python)."""
import os
import re

import numpy as np
import pytest

import paper_2508_06001_amd as K
from knap_inputs import table1_streams
from oracle import balancer as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = ""
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        assert header.endswith(".h"), header
        with open(os.path.join(ROOT, "include", header)) as f:
            text += f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(knap_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(K.EXPORTS)
    for name in declared:
        assert hasattr(K.lib, name), name


def test_attention_entry_points_reject_bad_arguments_without_touching_a_gpu():
    f = K.lib.knap_varlen_attn_fwd
    assert f(0, 0, 0, 0, 0, 2, 64, 0.125, 0, 0, 0) == K.KNAP_OK               # empty bag: nothing to do
    assert f(0, 0, 0, 0, 1, 2, 64, 0.125, 0, 0, 0) == K.KNAP_ERR_INVALID_ARG  # null pointers
    assert f(16, 16, 16, 16, 1, 2, 96, 0.125, 16, 16, 0) == K.KNAP_ERR_INVALID_ARG   # head dim
    assert f(16, 16, 16, 16, -1, 2, 64, 0.125, 16, 16, 0) == K.KNAP_ERR_INVALID_ARG
    assert f(16, 16, 16, 16, 1, 0, 64, 0.125, 16, 16, 0) == K.KNAP_ERR_INVALID_ARG
    assert f(8, 16, 16, 16, 1, 2, 64, 0.125, 16, 16, 0) == K.KNAP_ERR_INVALID_ARG    # misaligned q
    assert f(16, 16, 16, 16, K.KNAP_MAX_SEQS + 1, 2, 64, 0.125, 16, 16, 0) == K.KNAP_ERR_TOO_MANY_SEQS
    for bad_scale in (0.0, -0.125, float("inf"), float("nan")):
        assert f(16, 16, 16, 16, 1, 2, 64, bad_scale, 16, 16, 0) == K.KNAP_ERR_INVALID_ARG
    g = K.lib.knap_varlen_attn_bwd
    assert g(0, 0, 0, 0, 0, 2, 64, 0.125, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == K.KNAP_OK
    assert g(256, 512, 768, 1024, 1, 2, 64, 0.125, 1280, 1536, 1792, 2048, 2304, 2560, 100, 0, 0, 0) \
        == K.KNAP_ERR_INVALID_ARG          # no workspace
    need = K.knap_varlen_attn_bwd_workspace_bytes(100, 1, 2, 64)
    assert need >= 100 * 2 * 4
    assert g(256, 512, 768, 1024, 1, 2, 64, 0.125, 1280, 1536, 1792, 2048, 2304, 2560, 100, 4096, need - 1, 0) \
        == K.KNAP_ERR_WORKSPACE_TOO_SMALL
    assert K.knap_strerror(K.KNAP_ERR_WORKSPACE_TOO_SMALL) == "workspace too small"
    assert K.knap_strerror(12345) == "unknown error"


def test_workload_model_matches_oracle():
    for l in (1, 37, 452, 4292, 16580, 25796):
        assert K.knap_flux_workload(l, 3072, 0.49) == pytest.approx(B.flux_workload(l, 3072, 0.49), rel=1e-15)
        assert K.knap_seq_cost(l, 2.5e-9, 1.5e-6) == pytest.approx(B.seq_cost(l, 2.5e-9, 1.5e-6), rel=1e-15)


def test_topology_parser():
    assert K.knap_parse_topology("g1n2+g2n1+g4n1") == B.parse_topology("g1n2+g2n1+g4n1") == [1, 1, 2, 4]
    assert K.knap_parse_topology("g8n4") == [8] * 4
    assert K.knap_parse_topology(" g2n3 + g1n1 ") == [2, 2, 2, 1]
    for bad in ("", "g0n1", "g1n0", "x1n1", "g1n1+", "g1", "g1n1x"):
        with pytest.raises(K.KnapError) as e:
            K.knap_parse_topology(bad)
        assert e.value.code == K.KNAP_ERR_PARSE
    with pytest.raises(K.KnapError) as e:
        K.knap_parse_topology("g1n9", cap=4)
    assert e.value.code == K.KNAP_ERR_CAPACITY


@pytest.mark.parametrize("workload", ["low_res", "mixed_res", "joint"])
@pytest.mark.parametrize("topo", ["g1n32", "g2n16", "g4n8", "g8n4", "g1n2+g2n1+g4n1"])
def test_greedy_assignment_is_identical_to_oracle_on_table1_streams(workload, topo):
    for seed in (None, 0, 1):
        lens = [l for g in table1_streams(workload, seed) for l in g]
        w = [B.flux_workload(l, 3072, 0.49) for l in lens]
        bags = B.parse_topology(topo)
        bag_ref, load_ref = B.greedy_assign(w, bags)
        bag_c, load_c = K.knap_greedy_assign_weights(w, bags)
        assert bag_c == bag_ref                      # integer decisions: exact
        assert load_c == pytest.approx(load_ref, rel=1e-13)
        assert K.knap_wir(load_c, bags) == pytest.approx(B.wir(load_ref, bags), rel=1e-13)


def test_greedy_with_quadratic_cost_and_random_bags():
    rng = np.random.default_rng(5)
    for trial in range(20):
        n = int(rng.integers(1, 300))
        lens = [int(x) for x in rng.integers(0, 40000, size=n)]
        bags = [int(x) for x in rng.choice([1, 2, 4, 8], size=int(rng.integers(1, 9)))]
        a, b = 3.0e-9, 2.0e-6
        bag_ref, load_ref = B.greedy_assign([B.seq_cost(l, a, b) for l in lens], bags)
        bag_c, load_c = K.knap_greedy_assign(lens, bags, a, b)
        assert bag_c == bag_ref
        assert load_c == pytest.approx(load_ref, rel=1e-13)
        for j in range(len(bags)):
            got_len, got_cu = K.knap_bag_cu_seqlens(lens, bag_c, j)
            assert got_len == B.bag_sequences(lens, bag_ref, j)
            assert got_cu == [0] + list(np.cumsum(got_len))


def test_chunks_wir_and_fit():
    for L, g in ((10, 4), (8, 8), (16580, 8), (5, 8), (0, 3)):
        assert K.knap_chunk_lengths(L, g) == B.chunk_lengths(L, g)
    assert K.knap_wir([4.0, 6.0], [1, 2]) == pytest.approx(4.0 / 3.0)
    assert K.knap_wir([0.0, 6.0], [1, 2]) == float("inf")
    rng = np.random.default_rng(3)
    Ls = [rng.integers(200, 70000, size=int(rng.integers(1, 12))).astype(np.float64) for _ in range(25)]
    s2 = [float((x * x).sum()) for x in Ls]
    s1 = [float(x.sum()) for x in Ls]
    a, b = 1.7e-9, 3.3e-6
    t = [(a * x2 + b * x1) * (1.0 + 0.01 * rng.standard_normal()) for x2, x1 in zip(s2, s1)]
    got = K.knap_fit_cost_model(s2, s1, t)
    ref = B.fit_cost_model(s2, s1, t)
    assert got[0] == pytest.approx(ref[0], rel=1e-9)
    assert got[1] == pytest.approx(ref[1], rel=1e-9)
    assert got[2] == pytest.approx(ref[2], rel=1e-7)
    with pytest.raises(K.KnapError):
        K.knap_fit_cost_model([1.0], [1.0], [1.0])
    with pytest.raises(K.KnapError):
        K.knap_fit_cost_model([1.0, 2.0], [1.0, 2.0], [1.0, 0.0])


def test_ulysses_host_side_and_argument_checks():
    """Chunk bookkeeping of a multi-GPU bag against the oracle, and argument errors of the device entry
    points that are decided before anything touches a GPU."""
    from oracle import ulysses as U
    rng = np.random.default_rng(3)
    for g in (1, 2, 3, 8):
        lens = [int(v) for v in rng.integers(0, 5000, size=17)] + [0, 1, g - 1, g, g + 1]
        assert K.knap_ulysses_local_tokens(lens, g) == [U.local_tokens(lens, g, r) for r in range(g)]
        assert sum(K.knap_ulysses_local_tokens(lens, g)) == sum(lens)
    assert K.knap_ulysses_plan_workspace_bytes(10, 8) >= 11 * 8 * 4
    assert K.knap_ulysses_plan_workspace_bytes(-1, 8) == 0
    bad = K.KNAP_ERR_INVALID_ARG
    # H not divisible by g; a (token, head-group) row that is not a whole number of 16-byte units; g < 1
    assert K.lib.knap_ulysses_pack_heads(None, 16, 6, 64, 4, None, None) == bad
    assert K.lib.knap_ulysses_pack_heads(None, 16, 4, 4, 4, None, None) == bad
    assert K.lib.knap_ulysses_unpack_heads(None, 16, 8, 64, 0, None, None) == bad
    assert K.lib.knap_ulysses_gather_chunks(None, None, -1, 3, 128, None, None) == bad
    assert K.lib.knap_ulysses_plan(None, 4, 100, K.KNAP_ULYSSES_MAX_GPUS + 1, None, None, 0, None) == bad
    assert K.lib.knap_ulysses_plan(None, K.KNAP_MAX_SEQS + 1, 100, 8, None, None, 0, None) == K.KNAP_ERR_TOO_MANY_SEQS
    # nothing to do: success without pointers
    assert K.lib.knap_ulysses_pack_heads(None, 0, 8, 64, 4, None, None) == K.KNAP_OK
    assert K.lib.knap_ulysses_scatter_chunks(None, None, 0, 3, 128, None, None) == K.KNAP_OK
    assert K.lib.knap_ulysses_plan(None, 0, 0, 8, None, None, 0, None) == K.KNAP_OK


def test_table1_wir_script_reproduces_the_printed_column():
    """The user-facing reproduction (C balancer on the paper's data-code streams) stays in the bands of
    the cells the paper prints (the paper drew its own random streams)."""
    from paper_2508_06001_amd import table1_wir as T
    printed = T.printed_cells(os.path.join(ROOT, "tests", "golden", "table1_wir.txt"))
    assert len(printed) == 15
    assert T.printed_cells(None) == {}
    for (workload, topo), val in printed.items():
        got = float(np.median([T.wir(workload, topo, s) for s in range(5)]))
        if topo == "none":
            assert 0.5 * val <= got <= 1.6 * val, (workload, topo, got, val)
        else:
            assert abs(got - val) <= (0.6 if topo == "g1n32" else 0.12), (workload, topo, got, val)
