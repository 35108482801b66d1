"""Second workload: bags drawn from the paper's own simulator distributions (Sec. 4.1 data codes: text
U{0..392}, one aspect multiplier U[0.96, 1.04] per batch, (R/16)^2 visual tokens per frame, F/3.4 latent frames
for clips; the `joint` and `mixed_res` workloads of Table 1 on 32 GPUs), balanced into 32 one-GPU bags by the
greedy first pass of Sec. 3.3 with the Table 1 cost (Eq. 2, gamma = 0.49, d_model = 3072).  The bag lists are
formed by the ORACLE balancer (oracle/balancer.py) and the library's C balancer must agree with it; the
attention of the chosen bags then runs through the C ABI and is compared with the attention oracle, at the
FLUX shape (24 heads of 128) and at 48 heads of 64.  Same bars as tests/test_gpu_parity.py."""
import numpy as np
import pytest

import paper_2508_06001_amd as K
from knap_inputs import BagSpec, table1_streams
from oracle import attention as A
from oracle import balancer as B

from gpu_util import GpuRun, rel_fro, say
from test_gpu_parity import BWD_TOL, FWD_TOL, LSE_TOL, _invariants, _sampled_compare

pytestmark = pytest.mark.gpu

D_MODEL, GAMMA = 3072, 0.49


def _one_gpu_bags(workload: str, seed: int):
    pool = [L for g in table1_streams(workload, seed) for L in g]
    weights = [B.flux_workload(L, D_MODEL, GAMMA) for L in pool]
    bag_of, _ = B.greedy_assign(weights, [1] * 32)
    c_bag_of, _ = K.knap_greedy_assign_weights([K.knap_flux_workload(L, D_MODEL, GAMMA) for L in pool], [1] * 32)
    assert c_bag_of == bag_of                      # the library's balancer takes the same decisions
    bags = [B.bag_sequences(pool, bag_of, j) for j in range(32)]
    assert sorted(L for b in bags for L in b) == sorted(pool)
    return bags


@pytest.mark.timeout(300)
@pytest.mark.parametrize("H,d", [(24, 128), (48, 64)])
def test_joint_workload_bags(H, d):
    """`joint` (images 256..2048 px, key-frame sets, 85-frame clips): the bag holding the longest sequence (a
    512-px 85-frame clip, about 25.8k tokens) on sampled rows and key rows, and the bag with the most
    sequences against the full oracle on two heads."""
    bags = _one_gpu_bags("joint", seed=32)
    longest = max(range(32), key=lambda j: max(bags[j]))
    most = max(range(32), key=lambda j: len(bags[j]))
    assert max(bags[longest]) > 25000 and len(bags[most]) >= 4
    say(f"[sim] joint: longest bag {bags[longest]}, most sequences {bags[most]}")
    run = GpuRun(BagSpec("sim_joint_long", bags[longest], H=H, d=d, seed=9301 + d))
    s = int(np.argmax(bags[longest]))
    _sampled_compare(run, s, H // 2, n_rows=32, n_cols=16)
    _invariants(run, s, H - 1)
    run = GpuRun(BagSpec("sim_joint_many", bags[most], H=H, d=d, seed=9302 + d))
    cu = [int(c) for c in run.cu]
    for sq in range(len(bags[most])):
        for h in (0, H - 1):
            sl = slice(cu[sq], cu[sq + 1])
            Q, K_, V, dO = (run.host(n, sl, h) for n in ("q", "k", "v", "dout"))
            O, LSE = A.attn_fwd_dense(Q, K_, V, run.bag.scale)
            dQ, dK, dV = A.attn_bwd_dense(Q, K_, V, dO, run.bag.scale)
            assert float(np.max(np.abs(run.host("out", sl, h) - O))) <= FWD_TOL
            assert float(np.max(np.abs(run.lse[h, sl] - LSE))) <= LSE_TOL
            for name, ref in (("dq", dQ), ("dk", dK), ("dv", dV)):
                assert rel_fro(run.host(name, sl, h), ref) <= BWD_TOL, (name, sq, h)


@pytest.mark.timeout(300)
def test_mixed_res_workload_bag():
    """`mixed_res` (256..2048 px images): a bag that holds one 2048-px image (16384 visual tokens)."""
    bags = _one_gpu_bags("mixed_res", seed=31)
    j = max(range(32), key=lambda i: max(bags[i]))
    assert 16000 < max(bags[j]) < 18000
    run = GpuRun(BagSpec("sim_mixed_res", bags[j], H=24, d=128, seed=9311))
    s = int(np.argmax(bags[j]))
    _sampled_compare(run, s, 3, n_rows=32, n_cols=16)
    _invariants(run, s, 20)
