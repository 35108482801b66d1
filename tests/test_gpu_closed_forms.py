"""Full-size checks of EVERY element of every head on the benchmark bags 2, 3 and 4, from inputs whose exact
result follows from the definition of attention (Sec. 3.4 / attention listing of Sec. 3.5; Eq. 1) without an
L x L pass.  With one (sequence, head) of length L, P = softmax(scale Q K^T), O = P V, and for dO:
dV = P^T dO, dP = dO V^T, D_i = dO_i . O_i, dS = P (dP - D), dQ = scale dS K, dK = scale dS^T Q.

* K = 0: P_ij = 1/L.  O_i = mean(V), LSE_i = ln L, dV_j = sum_i dO_i / L, dQ = 0 (exactly: every term
  multiplies a zero K row), dK_j = (scale / L) A (V_j - mean(V)) with A = Q^T dO (d x d).
* Q = 0: P uniform as well.  dK = 0 exactly, dQ_i = (scale / L) (K^T V - L kbar vbar^T) dO_i.
* constant V rows (V_j = v): O = v bit for bit (v is a bf16 value and the weights sum to one), dP_ij = D_i
  for every j, so dS = 0 and dQ = dK = 0 up to float32 rounding of dP - D; sum_j dV_j = sum_i dO_i.
* causal mask with K = 0 or Q = 0: P_ij = 1/(i+1) for j <= i; O is the running mean of V, LSE_i = ln(i+1), and
  dQ, dK, dV follow from prefix and suffix sums (written out in causal_closed_forms.py, which the CPU suite
  checks against the oracle's causal mode): every element of the causal entry points' outputs on configs 2-4.
* periodic sequence: if q, k, v, dO of a sequence of length L = m p repeat with period p, every key of the
  period-p problem appears m times with the same score, so P_ij(L) = P_i'j'(p) / m and O, dQ, dK, dV of row
  i equal those of row i mod p of the period-p problem; LSE(L) = LSE(p) + ln m.  The period-p problem is
  evaluated by the float64 oracle; the 131072- and 65536-token sequences of configs 4 and 3 are thereby
  compared with it element by element, all heads, with a softmax that is not uniform.

The expected values are float64 torch expressions of the formulas above (or the oracle's output for the
period); none of them comes from the library.  A work item that the tile schedule dropped, doubled or gave
the wrong rows changes these results wherever it lies, which sampled rows cannot promise.
"""
import math

import numpy as np
import pytest

from knap_inputs import BagSpec, bf16_bits_to_f32, config_bag, cu_seqlens_of, make_qkv_dout
from oracle import attention as A

from causal_closed_forms import causal_zero_score_reference
from gpu_util import GpuRun, say

pytestmark = pytest.mark.gpu

FWD_TOL = 1e-2
LSE_TOL = 1e-3
BWD_TOL = 3e-2


def _randn_bf16(shape, seed):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)


def _rel(got, ref):
    import torch
    den = float(torch.linalg.vector_norm(ref))
    return float(torch.linalg.vector_norm(got - ref)) / (den if den > 0 else 1.0)


def _bags():
    return {2: config_bag(2), 3: config_bag(3), 4: config_bag(4)}


@pytest.mark.timeout(300)
@pytest.mark.parametrize("config", [2, 3, 4])
def test_zero_keys_every_element(config):
    import torch
    bag = _bags()[config]
    T, H, d = bag.total_tokens, bag.H, bag.d
    dev = {"q": _randn_bf16((T, H, d), bag.seed + 11), "k": torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda"),
           "v": _randn_bf16((T, H, d), bag.seed + 12), "dout": _randn_bf16((T, H, d), bag.seed + 13)}
    run = GpuRun(bag, device_tensors=dev)
    a = run.attn
    assert int(torch.count_nonzero(a.dq)) == 0                     # dQ = scale dS K with K = 0
    cu = [int(c) for c in run.cu]
    worst = {"out": 0.0, "lse": 0.0, "dv": 0.0, "dk": 0.0}
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        L = cu[s + 1] - cu[s]
        q, v, do = (dev[n][sl].double() for n in ("q", "v", "dout"))          # (L, H, d)
        vbar = v.mean(dim=0)                                                     # (H, d)
        worst["out"] = max(worst["out"], float((a.out[sl].double() - vbar).abs().max()))
        worst["lse"] = max(worst["lse"], float((a.lse[:, sl].double() - math.log(L)).abs().max()))
        dv_ref = (do.sum(dim=0) / L).expand(L, H, d)
        worst["dv"] = max(worst["dv"], _rel(a.dv[sl].double(), dv_ref))
        amat = torch.einsum("ihc,ihe->hce", q, do)                               # A = Q^T dO per head
        dk_ref = (bag.scale / L) * torch.einsum("hce,jhe->jhc", amat, v - vbar)
        worst["dk"] = max(worst["dk"], _rel(a.dk[sl].double(), dk_ref))
    say(f"[closed form] {bag.name} K=0: out {worst['out']:.3e} lse {worst['lse']:.3e} dv {worst['dv']:.3e} dk {worst['dk']:.3e}")
    assert worst["out"] <= FWD_TOL and worst["lse"] <= LSE_TOL
    assert worst["dv"] <= BWD_TOL and worst["dk"] <= BWD_TOL


@pytest.mark.timeout(300)
@pytest.mark.parametrize("config", [2, 3, 4])
def test_zero_queries_every_element(config):
    import torch
    bag = _bags()[config]
    T, H, d = bag.total_tokens, bag.H, bag.d
    dev = {"q": torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda"), "k": _randn_bf16((T, H, d), bag.seed + 21),
           "v": _randn_bf16((T, H, d), bag.seed + 22), "dout": _randn_bf16((T, H, d), bag.seed + 23)}
    run = GpuRun(bag, device_tensors=dev)
    a = run.attn
    assert int(torch.count_nonzero(a.dk)) == 0                     # dK = scale dS^T Q with Q = 0
    cu = [int(c) for c in run.cu]
    worst = {"out": 0.0, "lse": 0.0, "dv": 0.0, "dq": 0.0}
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        L = cu[s + 1] - cu[s]
        k, v, do = (dev[n][sl].double() for n in ("k", "v", "dout"))
        vbar, kbar = v.mean(dim=0), k.mean(dim=0)
        worst["out"] = max(worst["out"], float((a.out[sl].double() - vbar).abs().max()))
        worst["lse"] = max(worst["lse"], float((a.lse[:, sl].double() - math.log(L)).abs().max()))
        worst["dv"] = max(worst["dv"], _rel(a.dv[sl].double(), (do.sum(dim=0) / L).expand(L, H, d)))
        m = torch.einsum("jhc,jhe->hce", k, v) - L * torch.einsum("hc,he->hce", kbar, vbar)
        dq_ref = (bag.scale / L) * torch.einsum("hce,ihe->ihc", m, do)
        worst["dq"] = max(worst["dq"], _rel(a.dq[sl].double(), dq_ref))
    say(f"[closed form] {bag.name} Q=0: out {worst['out']:.3e} lse {worst['lse']:.3e} dv {worst['dv']:.3e} dq {worst['dq']:.3e}")
    assert worst["out"] <= FWD_TOL and worst["lse"] <= LSE_TOL
    assert worst["dv"] <= BWD_TOL and worst["dq"] <= BWD_TOL


@pytest.mark.timeout(300)
@pytest.mark.parametrize("config", [2, 3, 4])
def test_constant_value_rows_every_element(config):
    import torch
    bag = _bags()[config]
    T, H, d = bag.total_tokens, bag.H, bag.d
    cu = [int(c) for c in cu_seqlens_of(bag.seq_lens)]
    v_seq = _randn_bf16((len(bag.seq_lens), H, d), bag.seed + 32)               # one value row per (sequence, head)
    lens = torch.tensor(bag.seq_lens, device="cuda")
    v = torch.repeat_interleave(v_seq, lens, dim=0)
    k = _randn_bf16((T, H, d), bag.seed + 31)
    if bag.k_outlier_prob > 0:                                                   # the bag's peaky keys
        g = torch.Generator(device="cuda")
        g.manual_seed(bag.seed + 34)
        k = torch.where(torch.rand((T, H, d), generator=g, device="cuda") < bag.k_outlier_prob,
                        (k.float() * bag.k_outlier_scale).to(torch.bfloat16), k)
    dev = {"q": _randn_bf16((T, H, d), bag.seed + 30), "k": k, "v": v, "dout": _randn_bf16((T, H, d), bag.seed + 33)}
    run = GpuRun(bag, device_tensors=dev)
    a = run.attn
    assert torch.equal(a.out.view(torch.int16), v.view(torch.int16))            # O = v, bit for bit
    # dS = P (dP - D) vanishes but for the float32 rounding of dP - D (two summation orders of dO . v, each
    # good to about 1e-5 at |dO . v| ~ 11): dq and dk stay at that level, far below the size of ordinary
    # gradients of these bags (about 1e-1 and 1e-2)
    dq_max, dk_max = float(a.dq.float().abs().max()), float(a.dk.float().abs().max())
    worst = 0.0
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        lhs, rhs = a.dv[sl].double().sum(dim=0), dev["dout"][sl].double().sum(dim=0)
        scale_ = math.sqrt(float((a.dv[sl].double() ** 2).sum()) + float((dev["dout"][sl].double() ** 2).sum()))
        worst = max(worst, float(torch.linalg.vector_norm(lhs - rhs)) / scale_)
    say(f"[closed form] {bag.name} constant V: max|dq| {dq_max:.3e} max|dk| {dk_max:.3e} colsum(dv) {worst:.3e}")
    assert dq_max <= 1e-3 and dk_max <= 1e-3
    assert worst <= 2e-2


def _periodic_case(bag, s_long, period, seed):
    """Makes sequence s_long of the bag periodic with the given period, runs the library on the whole bag
    and compares every row of that sequence, all heads, with the oracle's result for one period."""
    import torch
    from paper_2508_06001_amd.runtime import bf16_bits_to_device, bf16_device_to_bits
    T, H, d = bag.total_tokens, bag.H, bag.d
    cu = [int(c) for c in cu_seqlens_of(bag.seq_lens)]
    L = bag.seq_lens[s_long]
    assert L % period == 0
    m = L // period
    small = BagSpec("period", [period], H=H, d=d, seed=seed, k_outlier_prob=bag.k_outlier_prob,
                    k_outlier_scale=bag.k_outlier_scale)
    bits = make_qkv_dout(small)
    dev = {}
    for i, n in enumerate(("q", "k", "v", "dout")):
        x = _randn_bf16((T, H, d), seed + 1 + i)
        x[cu[s_long]:cu[s_long + 1]] = bf16_bits_to_device(bits[n]).repeat(m, 1, 1)
        dev[n] = x
    run = GpuRun(bag, device_tensors=dev)
    a = run.attn
    sl = slice(cu[s_long], cu[s_long + 1])
    got = {n: bf16_bits_to_f32(bf16_device_to_bits(getattr(a, n)[sl])).astype(np.float64) for n in ("out", "dq", "dk", "dv")}
    lse = a.lse[:, sl].cpu().numpy().astype(np.float64)
    worst = {"out": 0.0, "lse": 0.0, "dq": 0.0, "dk": 0.0, "dv": 0.0}
    for h in range(H):
        Q, K_, V, dO = (bf16_bits_to_f32(bits[n][:, h, :]).astype(np.float64) for n in ("q", "k", "v", "dout"))
        O, LSE = A.attn_fwd_dense(Q, K_, V, bag.scale)
        ref = dict(zip(("dq", "dk", "dv"), A.attn_bwd_dense(Q, K_, V, dO, bag.scale)))
        err = np.abs(got["out"][:, h, :] - np.tile(O, (m, 1)))
        err = np.where(err <= 2.0 ** -8 * np.abs(np.tile(O, (m, 1))), 0.0, err) if bag.k_outlier_prob > 0 else err
        worst["out"] = max(worst["out"], float(err.max()))
        worst["lse"] = max(worst["lse"], float(np.abs(lse[h] - np.tile(LSE + math.log(m), m)).max()))
        for n in ("dq", "dk", "dv"):
            r = np.tile(ref[n], (m, 1))
            worst[n] = max(worst[n], float(np.linalg.norm(got[n][:, h, :] - r) / np.linalg.norm(r)))
            # and tile by tile: no 128-row block of the long sequence may be off by more than the bar either
            blocks = (got[n][:, h, :] - r).reshape(L // 128, -1)
            rb = r.reshape(L // 128, -1)
            worst[n] = max(worst[n], float((np.linalg.norm(blocks, axis=1) / np.linalg.norm(rb, axis=1)).max()))
    say(f"[periodic] {bag.name} seq {s_long} L={L} period {period}: " + " ".join(f"{k} {v:.3e}" for k, v in worst.items()))
    assert worst["out"] <= FWD_TOL
    assert worst["lse"] <= (3e-3 if bag.k_outlier_prob > 0 else LSE_TOL)
    for n in ("dq", "dk", "dv"):
        assert worst[n] <= BWD_TOL, (n, worst[n])


@pytest.mark.timeout(300)
def test_periodic_131072_token_sequence_every_element():
    """Config 4 (H = 3): the 131072-token sequence repeats a 1024-token period 128 times."""
    _periodic_case(config_bag(4), 0, 1024, seed=7171)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("long_position", ["middle", "last"])
def test_periodic_65536_token_sequence_every_element(long_position):
    """Config 3 (H = 24, peaky keys, 200 short sequences around it): the 65536-token sequence repeats a
    2048-token period 32 times."""
    bag = config_bag(3, long_position=long_position)
    _periodic_case(bag, bag.seq_lens.index(65536), 2048, seed=7272)


@pytest.mark.timeout(300)
def test_periodic_sequence_with_a_period_that_no_tile_divides():
    """Period 1031 (prime) x 127 repeats = 130937 tokens: the period boundaries fall inside tiles and the
    sequence ends in a ragged tile."""
    bag = BagSpec("periodic_prime", [130937, 5000], H=2, d=128, seed=7373)
    import torch  # noqa: F401
    T, H, d = bag.total_tokens, bag.H, bag.d
    period, m, L = 1031, 127, 130937
    small = BagSpec("period", [period], H=H, d=d, seed=7374)
    bits = make_qkv_dout(small)
    from paper_2508_06001_amd.runtime import bf16_bits_to_device, bf16_device_to_bits
    dev = {}
    for i, n in enumerate(("q", "k", "v", "dout")):
        x = _randn_bf16((T, H, d), 7375 + i)
        x[:L] = bf16_bits_to_device(bits[n]).repeat(m, 1, 1)
        dev[n] = x
    run = GpuRun(bag, device_tensors=dev)
    a = run.attn
    got = {n: bf16_bits_to_f32(bf16_device_to_bits(getattr(a, n)[:L])).astype(np.float64) for n in ("out", "dq", "dk", "dv")}
    lse = a.lse[:, :L].cpu().numpy().astype(np.float64)
    for h in range(H):
        Q, K_, V, dO = (bf16_bits_to_f32(bits[n][:, h, :]).astype(np.float64) for n in ("q", "k", "v", "dout"))
        O, LSE = A.attn_fwd_dense(Q, K_, V, bag.scale)
        ref = dict(zip(("dq", "dk", "dv"), A.attn_bwd_dense(Q, K_, V, dO, bag.scale)))
        e_out = float(np.abs(got["out"][:, h, :] - np.tile(O, (m, 1))).max())
        e_lse = float(np.abs(lse[h] - np.tile(LSE + math.log(m), m)).max())
        errs = {n: float(np.linalg.norm(got[n][:, h, :] - np.tile(ref[n], (m, 1))) / np.linalg.norm(np.tile(ref[n], (m, 1))))
                for n in ("dq", "dk", "dv")}
        say(f"[periodic] prime period head {h}: out {e_out:.3e} lse {e_lse:.3e} " + " ".join(f"{k} {v:.3e}" for k, v in errs.items()))
        assert e_out <= FWD_TOL and e_lse <= LSE_TOL
        for n in errs:
            assert errs[n] <= BWD_TOL, (n, errs[n])


@pytest.mark.timeout(400)
@pytest.mark.parametrize("zero", ["k", "q"])
@pytest.mark.parametrize("config", [2, 3, 4])
def test_causal_zero_scores_every_element(config, zero):
    """The causal entry points at full size with K = 0 (or Q = 0): every row of every head against the closed
    form.  The first rows of a sequence see one or two keys and return single v entries, so the forward bar
    is relative there (2^-8 |ref|, one bf16 rounding)."""
    import torch
    bag = _bags()[config]
    T, H, d = bag.total_tokens, bag.H, bag.d
    dev = {n: _randn_bf16((T, H, d), bag.seed + 40 + i) for i, n in enumerate(("q", "k", "v", "dout"))}
    dev[zero] = torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda")
    run = GpuRun(bag, device_tensors=dev, causal=True)
    a = run.attn
    assert int(torch.count_nonzero(a.dq if zero == "k" else a.dk)) == 0     # every term multiplies a zero row
    cu = [int(c) for c in run.cu]
    worst = {"out": 0.0, "lse": 0.0, "dq": 0.0, "dk": 0.0, "dv": 0.0}
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        q, k, v, do = (dev[n][sl].double() for n in ("q", "k", "v", "dout"))
        out, lse, dq, dk, dv = causal_zero_score_reference(q, k, v, do, bag.scale)
        err = (a.out[sl].double() - out).abs()
        err = torch.where(err <= 2.0 ** -8 * out.abs(), torch.zeros_like(err), err)
        worst["out"] = max(worst["out"], float(err.max()))
        worst["lse"] = max(worst["lse"], float((a.lse[:, sl].double() - lse).abs().max()))
        worst["dv"] = max(worst["dv"], _rel(a.dv[sl].double(), dv))
        if zero == "k":
            worst["dk"] = max(worst["dk"], _rel(a.dk[sl].double(), dk))
        else:
            worst["dq"] = max(worst["dq"], _rel(a.dq[sl].double(), dq))
        del q, k, v, do, out, lse, dq, dk, dv, err
    say(f"[closed form] {bag.name} causal {zero.upper()}=0: " + " ".join(f"{n} {e:.3e}" for n, e in worst.items()))
    assert worst["out"] <= FWD_TOL and worst["lse"] <= LSE_TOL
    for n in ("dq", "dk", "dv"):
        assert worst[n] <= BWD_TOL, (n, worst[n])
