"""Pins of the causal mode of the attention oracle (the second homogeneous mask
the paper admits inside a datum, Limitations paragraph) against things other
than itself:

* scalar-loop brute force over the packed T x T problem with the mask written
  out element by element;
* closed forms: row 0 sees one key; zero K gives running means and
  LSE_i = ln(i + 1); constant V; the last row equals the unmasked last row;
* the prefix property: the first n rows do not depend on anything after them;
* central finite differences of sum(dO * O);
* torch float64 softmax with an explicit lower-triangular mask + autograd;
* sampled rows / columns against the full evaluation; invariants;
* planted mistakes (strict mask, transposed mask) must break a closed form.
"""
import math

import numpy as np
import pytest

from knap_inputs import cu_seqlens_of
from oracle import attention as A


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _brute_force_packed_causal(q, k, v, dout, cu, scale):
    """Pure-Python scalar loops; key j is visible to query i iff same sequence and j <= i."""
    T, H, d = q.shape
    seq_of = [0] * T
    for s in range(len(cu) - 1):
        for r in range(cu[s], cu[s + 1]):
            seq_of[r] = s
    out, dq, dk, dv = (np.zeros((T, H, d)) for _ in range(4))
    lse = np.zeros((H, T))
    for h in range(H):
        for i in range(T):
            vis = [j for j in range(T) if seq_of[j] == seq_of[i] and j <= i]
            s_row = [scale * math.fsum(float(q[i, h, c]) * float(k[j, h, c]) for c in range(d)) for j in vis]
            m = max(s_row)
            e = [math.exp(x - m) for x in s_row]
            z = math.fsum(e)
            p = [x / z for x in e]
            lse[h, i] = m + math.log(z)
            for c in range(d):
                out[i, h, c] = math.fsum(pj * float(v[j, h, c]) for pj, j in zip(p, vis))
            dP = [math.fsum(float(dout[i, h, c]) * float(v[j, h, c]) for c in range(d)) for j in vis]
            delta = math.fsum(pj * x for pj, x in zip(p, dP))
            dS = [pj * (x - delta) for pj, x in zip(p, dP)]
            for c in range(d):
                dq[i, h, c] = scale * math.fsum(ds * float(k[j, h, c]) for ds, j in zip(dS, vis))
            for ds, pj, j in zip(dS, p, vis):
                for c in range(d):
                    dk[j, h, c] += scale * ds * float(q[i, h, c])
                    dv[j, h, c] += pj * float(dout[i, h, c])
    return out, lse, dq, dk, dv


def test_brute_force_packed_tiny_causal():
    rng = np.random.default_rng(21)
    lens = [3, 1, 6, 0, 4]
    cu = [int(x) for x in cu_seqlens_of(lens)]
    T, H, d = cu[-1], 2, 4
    q, k, v, do = (_rand(rng, T, H, d) for _ in range(4))
    scale = 0.41
    ref = _brute_force_packed_causal(q, k, v, do, cu, scale)
    o, lse = A.varlen_attn_fwd(q, k, v, cu, scale, causal=True)
    dq, dk, dv = A.varlen_attn_bwd(q, k, v, cu, scale, do, causal=True)
    for a, b in zip(ref, (o, lse, dq, dk, dv)):
        assert np.max(np.abs(a - b)) <= 1e-12
    # and it is not the unmasked result
    o_full, _ = A.varlen_attn_fwd(q, k, v, cu, scale)
    assert np.max(np.abs(o - o_full)) > 1e-2


def test_first_row_sees_one_key_and_last_row_sees_all():
    rng = np.random.default_rng(22)
    L, d = 19, 6
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 0.3
    O, LSE = A.attn_fwd_dense(Q, K, V, scale, causal=True)
    assert np.max(np.abs(O[0] - V[0])) <= 1e-15
    assert abs(LSE[0] - scale * Q[0] @ K[0]) <= 1e-14
    O_full, LSE_full = A.attn_fwd_dense(Q, K, V, scale)
    assert np.max(np.abs(O[-1] - O_full[-1])) <= 1e-14 and abs(LSE[-1] - LSE_full[-1]) <= 1e-14
    # with only the last row's dO non-zero, the whole backward equals the unmasked one
    dO_last = np.zeros_like(dO)
    dO_last[-1] = dO[-1]
    g_c = A.attn_bwd_dense(Q, K, V, dO_last, scale, causal=True)
    g_f = A.attn_bwd_dense(Q, K, V, dO_last, scale)
    for a, b in zip(g_c, g_f):
        assert np.max(np.abs(a - b)) <= 1e-13


def test_zero_k_gives_running_means():
    rng = np.random.default_rng(23)
    L, d = 17, 5
    Q, V, dO = (_rand(rng, L, d) for _ in range(3))
    K = np.zeros((L, d))
    O, LSE = A.attn_fwd_dense(Q, K, V, 0.8, causal=True)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.8, causal=True)
    n = np.arange(1, L + 1)
    assert np.max(np.abs(O - np.cumsum(V, axis=0) / n[:, None])) <= 1e-14
    assert np.max(np.abs(LSE - np.log(n))) <= 1e-14
    # dV_j = sum over i >= j of dO_i / (i + 1): a reversed running sum
    w = dO / n[:, None]
    assert np.max(np.abs(dV - np.cumsum(w[::-1], axis=0)[::-1])) <= 1e-14
    assert np.max(np.abs(dQ)) <= 1e-15


def test_constant_v_gives_v_and_zero_dq_dk_causal():
    rng = np.random.default_rng(24)
    L, d = 21, 7
    Q, K, dO = (_rand(rng, L, d) for _ in range(3))
    V = np.tile(_rand(rng, 1, d), (L, 1))
    O, _ = A.attn_fwd_dense(Q, K, V, 0.5, causal=True)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.5, causal=True)
    assert np.max(np.abs(O - V)) <= 1e-14
    assert np.max(np.abs(dQ)) <= 1e-13 and np.max(np.abs(dK)) <= 1e-13
    assert np.max(np.abs(dV.sum(axis=0) - dO.sum(axis=0))) <= 1e-13


def test_prefix_property():
    """Rows 0..n-1 of a causal sequence are the causal result of the n-row prefix alone."""
    rng = np.random.default_rng(25)
    L, n, d = 30, 11, 4
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    O, LSE = A.attn_fwd_dense(Q, K, V, 0.45, causal=True)
    Op, LSEp = A.attn_fwd_dense(Q[:n], K[:n], V[:n], 0.45, causal=True)
    assert np.max(np.abs(O[:n] - Op)) <= 1e-14 and np.max(np.abs(LSE[:n] - LSEp)) <= 1e-14
    # a loss that reads only the prefix rows has no gradient after the prefix
    dOp = dO.copy()
    dOp[n:] = 0.0
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dOp, 0.45, causal=True)
    dQp, dKp, dVp = A.attn_bwd_dense(Q[:n], K[:n], V[:n], dO[:n], 0.45, causal=True)
    for a, b in ((dQ, dQp), (dK, dKp), (dV, dVp)):
        assert np.max(np.abs(a[:n] - b)) <= 1e-13
        assert np.max(np.abs(a[n:])) == 0.0


def test_finite_differences_causal():
    rng = np.random.default_rng(26)
    lens = [4, 6]
    cu = [int(x) for x in cu_seqlens_of(lens)]
    T, H, d = cu[-1], 2, 3
    q, k, v, do = (_rand(rng, T, H, d) for _ in range(4))
    scale = 0.55
    grads = A.varlen_attn_bwd(q, k, v, cu, scale, do, causal=True)

    def f(qq, kk, vv):
        o, _ = A.varlen_attn_fwd(qq, kk, vv, cu, scale, causal=True)
        return float((o * do).sum())

    eps = 1e-6
    xs = [q, k, v]
    for which, g in enumerate(grads):
        num = np.zeros_like(g)
        it = np.nditer(xs[which], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args_p = [x.copy() for x in xs]
            args_m = [x.copy() for x in xs]
            args_p[which][idx] += eps
            args_m[which][idx] -= eps
            num[idx] = (f(*args_p) - f(*args_m)) / (2 * eps)
        rel = np.linalg.norm(num - g) / np.linalg.norm(g)
        assert rel <= 1e-6, (which, rel)


def test_single_sequence_matches_torch_float64_autograd_causal():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(27)
    L, d = 53, 16
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 1.0 / math.sqrt(d)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    S = (tq @ tk.T) * scale
    S = S.masked_fill(torch.ones(L, L, dtype=torch.bool).triu(1), float("-inf"))
    o = torch.softmax(S, dim=-1) @ tv
    (o * torch.tensor(dO)).sum().backward()
    O, LSE = A.attn_fwd_dense(Q, K, V, scale, causal=True)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, scale, causal=True)
    assert np.max(np.abs(O - o.detach().numpy())) <= 1e-13
    assert np.max(np.abs(LSE - torch.logsumexp(S, dim=-1).detach().numpy())) <= 1e-13
    assert np.max(np.abs(dQ - tq.grad.numpy())) <= 1e-12
    assert np.max(np.abs(dK - tk.grad.numpy())) <= 1e-12
    assert np.max(np.abs(dV - tv.grad.numpy())) <= 1e-12


def test_invariants_blocking_and_sampling_causal(monkeypatch):
    rng = np.random.default_rng(28)
    L, d = 47, 8
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 0.35
    O, LSE = A.attn_fwd_dense(Q, K, V, scale, causal=True)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, scale, causal=True)
    assert np.max(np.abs(dV.sum(axis=0) - dO.sum(axis=0))) <= 1e-12      # rows of P still sum to one
    assert abs((Q * dQ).sum() - (K * dK).sum()) <= 1e-11
    rows = [0, 5, 46, 20]
    o_r, lse_r, dq_r = A.attn_query_rows(Q, K, V, dO, rows, scale, causal=True)
    assert np.max(np.abs(o_r - O[rows])) <= 1e-13
    assert np.max(np.abs(lse_r - LSE[rows])) <= 1e-13
    assert np.max(np.abs(dq_r - dQ[rows])) <= 1e-12
    cols = [46, 0, 17]
    dk_c, dv_c = A.attn_key_cols(Q, K, V, dO, cols, scale, causal=True)
    assert np.max(np.abs(dk_c - dK[cols])) <= 1e-12
    assert np.max(np.abs(dv_c - dV[cols])) <= 1e-12
    monkeypatch.setattr(A, "_ROW_BLOCK_BYTES", 8 * L * 5)   # 5 rows at a time: the mask must follow the block offset
    O2, LSE2 = A.attn_fwd_dense(Q, K, V, scale, causal=True)
    g2 = A.attn_bwd_dense(Q, K, V, dO, scale, causal=True)
    assert np.max(np.abs(O - O2)) <= 1e-12 and np.max(np.abs(LSE - LSE2)) <= 1e-12
    for a, b in zip((dQ, dK, dV), g2):
        assert np.max(np.abs(a - b)) <= 1e-12


@pytest.mark.parametrize("mutation", ["strict_mask", "transposed_mask", "mask_ignores_block_offset"])
def test_closed_forms_catch_planted_mask_mistakes(mutation):
    """A wrong mask in a copy of the forward must break the zero-K closed form LSE_i = ln(i + 1)."""
    L = 9
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    if mutation == "strict_mask":
        hidden = j >= i
    elif mutation == "transposed_mask":
        hidden = j < i
    else:
        hidden = j > (i % 4)                       # rows counted from the start of a 4-row block
    S = np.where(hidden, -np.inf, 0.0)
    with np.errstate(invalid="ignore", divide="ignore"):
        lse = np.log(np.exp(S).sum(axis=1))
    assert not np.allclose(lse, np.log(np.arange(1, L + 1)))
