"""The benchmark's FLOP accounting (no GPU): forward 4, dK/dV kernel 8, dQ kernel 2 units of H d sum(L^2);
under the causal mask the score pairs are L (L + 1) / 2 per sequence; --gpus above 1 is refused."""
import os
import subprocess
import sys

import bench
from knap_inputs import BagSpec, config_bag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_flop_split_adds_up_to_fourteen():
    bag = config_bag(0)
    unit = bag.H * bag.d * sum(L * L for L in bag.seq_lens)
    assert bench.flops_fwd(bag) == 4.0 * unit
    assert bench.flops_bwd(bag) == 10.0 * unit
    assert bench.flops_dkdv_kernel(bag) == 8.0 * unit
    assert bench.flops_fwd(bag) + bench.flops_bwd(bag) == 14.0 * unit


def test_causal_counts_visible_pairs_only():
    bag = BagSpec("t", [1, 2, 5, 0], H=3, d=64, seed=1)
    assert bench.score_count(bag) == 1 + 4 + 25
    assert bench.score_count(bag, causal=True) == 1 + 3 + 15
    assert bench.flops_fwd(bag, True) == 4.0 * 3 * 64 * 19


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "--gpus must be 1" in p.stderr


def test_tile_padded_score_count():
    assert bench.tile_padded_sum_l2([256, 512, 1024]) == float(256 ** 2 + 512 ** 2 + 1024 ** 2)
    # 100 tokens: one 128-row query tile (10/18 of the work) and one 256-row key tile (8/18)
    assert abs(bench.tile_padded_sum_l2([100]) - 100 * (10 / 18 * 128 + 8 / 18 * 256)) < 1e-9
    assert bench.tile_padded_sum_l2([300]) > 300.0 ** 2
