"""Pins of the attention oracle against things other than itself.

Every check here is chosen so that a plausible mistake in oracle/attention.py
(dropped scale, wrong sign in dS, transposed operand, attention leaking across
sequences, wrong LSE) fails at least one of them:

* scalar-loop brute force over the packed T x T masked problem (no numpy
  matmul, no per-sequence slicing);
* dense masked numpy evaluation at the size of the tiny benchmark bag;
* closed forms: constant V, zero K, L = 1, one dominant key;
* central finite differences of sum(dO * O);
* torch float64 softmax attention + autograd on one sequence (library case);
* algebraic invariants of the backward.
"""
import math

import numpy as np
import pytest

from knap_inputs import bf16_bits_to_f32, config_bag, cu_seqlens_of, make_qkv_dout
from oracle import attention as A


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ----------------------------------------------------------------- brute force

def _brute_force_packed(q, k, v, dout, cu, scale):
    """Pure-Python scalar loops on the packed problem with a block-diagonal mask."""
    T, H, d = q.shape
    seq_of = [0] * T
    for s in range(len(cu) - 1):
        for r in range(cu[s], cu[s + 1]):
            seq_of[r] = s
    out = np.zeros((T, H, d))
    lse = np.zeros((H, T))
    dq = np.zeros((T, H, d))
    dk = np.zeros((T, H, d))
    dv = np.zeros((T, H, d))
    for h in range(H):
        P = [[0.0] * T for _ in range(T)]
        for i in range(T):
            s_row = []
            for j in range(T):
                if seq_of[i] != seq_of[j]:
                    s_row.append(-math.inf)
                else:
                    acc = 0.0
                    for c in range(d):
                        acc += float(q[i, h, c]) * float(k[j, h, c])
                    s_row.append(scale * acc)
            m = max(s_row)
            e = [math.exp(x - m) for x in s_row]
            z = math.fsum(e)
            lse[h, i] = m + math.log(z)
            for j in range(T):
                P[i][j] = e[j] / z
            for c in range(d):
                out[i, h, c] = math.fsum(P[i][j] * float(v[j, h, c]) for j in range(T))
        for i in range(T):
            dP = [math.fsum(float(dout[i, h, c]) * float(v[j, h, c]) for c in range(d)) for j in range(T)]
            delta = math.fsum(P[i][j] * dP[j] for j in range(T))
            dS = [P[i][j] * (dP[j] - delta) for j in range(T)]
            for c in range(d):
                dq[i, h, c] = scale * math.fsum(dS[j] * float(k[j, h, c]) for j in range(T))
            for j in range(T):
                if P[i][j] == 0.0:
                    continue
                for c in range(d):
                    dk[j, h, c] += scale * dS[j] * float(q[i, h, c])
                    dv[j, h, c] += P[i][j] * float(dout[i, h, c])
    return out, lse, dq, dk, dv


def test_brute_force_packed_tiny():
    rng = np.random.default_rng(1)
    lens = [3, 1, 5, 0, 4]
    cu = [int(x) for x in cu_seqlens_of(lens)]
    T, H, d = cu[-1], 2, 4
    q, k, v, do = (_rand(rng, T, H, d) for _ in range(4))
    scale = 0.37
    out, lse, dq, dk, dv = _brute_force_packed(q, k, v, do, cu, scale)
    o2, l2 = A.varlen_attn_fwd(q, k, v, cu, scale)
    dq2, dk2, dv2 = A.varlen_attn_bwd(q, k, v, cu, scale, do)
    for a, b in ((out, o2), (lse, l2), (dq, dq2), (dk, dk2), (dv, dv2)):
        assert np.max(np.abs(a - b)) <= 1e-12


def test_dense_masked_at_tiny_bag_size():
    """Packed output equals a whole-row softmax over a T x T block-diagonal mask."""
    bag = config_bag(0)
    t = make_qkv_dout(bag)
    q, k, v, do = (bf16_bits_to_f32(t[n]).astype(np.float64) for n in ("q", "k", "v", "dout"))
    cu = cu_seqlens_of(bag.seq_lens)
    T = bag.total_tokens
    seq_id = np.repeat(np.arange(len(bag.seq_lens)), bag.seq_lens)
    mask = seq_id[:, None] == seq_id[None, :]
    o_ref = np.zeros_like(q)
    lse_ref = np.zeros((bag.H, T))
    dq_ref, dk_ref, dv_ref = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    for h in range(bag.H):
        S = np.einsum("ic,jc->ij", q[:, h], k[:, h]) * bag.scale
        S = np.where(mask, S, -np.inf)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        Z = E.sum(axis=1, keepdims=True)
        P = E / Z
        lse_ref[h] = (m + np.log(Z))[:, 0]
        o_ref[:, h] = np.einsum("ij,jc->ic", P, v[:, h])
        dP = np.einsum("ic,jc->ij", do[:, h], v[:, h])
        dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
        dq_ref[:, h] = bag.scale * np.einsum("ij,jc->ic", dS, k[:, h])
        dk_ref[:, h] = bag.scale * np.einsum("ij,ic->jc", dS, q[:, h])
        dv_ref[:, h] = np.einsum("ij,ic->jc", P, do[:, h])
    o, lse = A.varlen_attn_fwd(q, k, v, cu, bag.scale)
    dq, dk, dv = A.varlen_attn_bwd(q, k, v, cu, bag.scale, do)
    assert np.max(np.abs(o - o_ref)) <= 1e-12
    assert np.max(np.abs(lse - lse_ref)) <= 1e-12
    for a, b in ((dq, dq_ref), (dk, dk_ref), (dv, dv_ref)):
        assert np.max(np.abs(a - b)) <= 1e-11


# ----------------------------------------------------------------- closed forms

def test_constant_v_gives_v_and_zero_dq_dk():
    rng = np.random.default_rng(2)
    L, d = 23, 8
    Q, K, dO = _rand(rng, L, d), _rand(rng, L, d), _rand(rng, L, d)
    row = _rand(rng, d)
    V = np.tile(row, (L, 1))
    O, _ = A.attn_fwd_dense(Q, K, V, 0.3)
    assert np.max(np.abs(O - V)) <= 1e-13
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.3)
    assert np.max(np.abs(dQ)) <= 1e-13 and np.max(np.abs(dK)) <= 1e-13
    # dV_j = sum_i P_ij dO_i: its column sum equals the column sum of dO
    assert np.max(np.abs(dV.sum(axis=0) - dO.sum(axis=0))) <= 1e-12


def test_zero_k_is_uniform_attention():
    rng = np.random.default_rng(3)
    L, d = 17, 6
    Q, V, dO = _rand(rng, L, d), _rand(rng, L, d), _rand(rng, L, d)
    K = np.zeros((L, d))
    O, LSE = A.attn_fwd_dense(Q, K, V, 0.5)
    assert np.max(np.abs(O - V.mean(axis=0, keepdims=True))) <= 1e-13
    assert np.max(np.abs(LSE - math.log(L))) <= 1e-13
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.5)
    assert np.max(np.abs(dQ)) <= 1e-13
    assert np.max(np.abs(dV - dO.sum(axis=0, keepdims=True) / L)) <= 1e-13
    # dK_j = scale * (1/L) * sum_i (dO_i . (V_j - mean V)) Q_i
    Vc = V - V.mean(axis=0, keepdims=True)
    dK_ref = 0.5 / L * (dO @ Vc.T).T @ Q
    assert np.max(np.abs(dK - dK_ref)) <= 1e-12


def test_length_one_sequence():
    rng = np.random.default_rng(4)
    d = 8
    Q, K, V, dO = (_rand(rng, 1, d) for _ in range(4))
    O, LSE = A.attn_fwd_dense(Q, K, V, 0.25)
    assert np.array_equal(O, V)
    assert abs(LSE[0] - 0.25 * float(Q[0] @ K[0])) <= 1e-14
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.25)
    assert np.array_equal(dV, dO)
    assert np.max(np.abs(dQ)) == 0.0 and np.max(np.abs(dK)) == 0.0


def test_one_dominant_key_selects_its_value():
    rng = np.random.default_rng(5)
    L, d = 9, 4
    Q = np.abs(_rand(rng, L, d)) + 0.5
    K = _rand(rng, L, d) * 0.01
    K[3] = 200.0          # q . k_3 is huge and positive for every query
    V = _rand(rng, L, d)
    O, _ = A.attn_fwd_dense(Q, K, V, 1.0)
    assert np.max(np.abs(O - V[3][None, :])) <= 1e-12


# ----------------------------------------------------------------- finite differences

def test_finite_differences():
    rng = np.random.default_rng(6)
    lens = [5, 7]
    cu = [int(x) for x in cu_seqlens_of(lens)]
    T, H, d = cu[-1], 2, 3
    q, k, v, do = (_rand(rng, T, H, d) for _ in range(4))
    scale = 0.6
    dq, dk, dv = A.varlen_attn_bwd(q, k, v, cu, scale, do)

    def f(qq, kk, vv):
        o, _ = A.varlen_attn_fwd(qq, kk, vv, cu, scale)
        return float((o * do).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num[idx] = (f(*args_p) - f(*args_m)) / (2 * eps)
        rel = np.linalg.norm(num - g) / np.linalg.norm(g)
        assert rel <= 1e-6, (name, rel)


# ----------------------------------------------------------------- library special case

def test_single_sequence_matches_torch_float64_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    L, d = 61, 16
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 1.0 / math.sqrt(d)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    S = (tq @ tk.T) * scale
    o = torch.softmax(S, dim=-1) @ tv
    (o * torch.tensor(dO)).sum().backward()
    O, LSE = A.attn_fwd_dense(Q, K, V, scale)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, scale)
    assert np.max(np.abs(O - o.detach().numpy())) <= 1e-13
    assert np.max(np.abs(LSE - torch.logsumexp(S, dim=-1).detach().numpy())) <= 1e-13
    assert np.max(np.abs(dQ - tq.grad.numpy())) <= 1e-12
    assert np.max(np.abs(dK - tk.grad.numpy())) <= 1e-12
    assert np.max(np.abs(dV - tv.grad.numpy())) <= 1e-12


# ----------------------------------------------------------------- invariants

def test_backward_invariants_and_symmetries():
    rng = np.random.default_rng(8)
    L, d = 40, 8
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 0.4
    O, LSE = A.attn_fwd_dense(Q, K, V, scale)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, scale)
    # softmax rows sum to one, seen through the backward
    assert np.max(np.abs(dV.sum(axis=0) - dO.sum(axis=0))) <= 1e-12
    # <Q, dQ> = <K, dK> (both are scale * sum_ij dS_ij q_i.k_j)
    assert abs((Q * dQ).sum() - (K * dK).sum()) <= 1e-11
    # LSE is the log of the row sum of exp(S)
    S = scale * Q @ K.T
    assert np.max(np.abs(np.exp(S - LSE[:, None]).sum(axis=1) - 1.0)) <= 1e-13
    # permuting keys/values: O unchanged, dK and dV permuted
    perm = rng.permutation(L)
    O2, _ = A.attn_fwd_dense(Q, K[perm], V[perm], scale)
    dQ2, dK2, dV2 = A.attn_bwd_dense(Q, K[perm], V[perm], dO, scale)
    assert np.max(np.abs(O - O2)) <= 1e-13
    assert np.max(np.abs(dK[perm] - dK2)) <= 1e-12 and np.max(np.abs(dV[perm] - dV2)) <= 1e-12
    # adding one vector to every key shifts each score row by a constant
    shift = _rand(rng, d)
    O3, LSE3 = A.attn_fwd_dense(Q, K + shift, V, scale)
    dQ3, _, dV3 = A.attn_bwd_dense(Q, K + shift, V, dO, scale)
    assert np.max(np.abs(O - O3)) <= 1e-12
    assert np.max(np.abs(LSE3 - (LSE + scale * Q @ shift))) <= 1e-12
    assert np.max(np.abs(dQ - dQ3)) <= 1e-11 and np.max(np.abs(dV - dV3)) <= 1e-12


def test_sequences_are_independent():
    rng = np.random.default_rng(9)
    lens = [6, 11, 4]
    cu = [int(x) for x in cu_seqlens_of(lens)]
    T, H, d = cu[-1], 2, 4
    q, k, v, do = (_rand(rng, T, H, d) for _ in range(4))
    o, lse = A.varlen_attn_fwd(q, k, v, cu, 0.5)
    dq, dk, dv = A.varlen_attn_bwd(q, k, v, cu, 0.5, do)
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    for x in (q2, k2, v2, do2):          # change the middle sequence only
        x[cu[1]:cu[2]] = _rand(rng, lens[1], H, d)
    o2, lse2 = A.varlen_attn_fwd(q2, k2, v2, cu, 0.5)
    dq2, dk2, dv2 = A.varlen_attn_bwd(q2, k2, v2, cu, 0.5, do2)
    keep = np.r_[0:cu[1], cu[2]:T]
    for a, b in ((o, o2), (dq, dq2), (dk, dk2), (dv, dv2)):
        assert np.array_equal(a[keep], b[keep])
    assert np.array_equal(lse[:, keep], lse2[:, keep])
    # and the packed result equals running each sequence alone
    for s in range(3):
        sl = slice(cu[s], cu[s + 1])
        for h in range(H):
            O, L_ = A.attn_fwd_dense(q[sl, h], k[sl, h], v[sl, h], 0.5)
            assert np.array_equal(O, o[sl, h]) and np.array_equal(L_, lse[h, sl])


def test_row_blocked_evaluation_equals_unblocked(monkeypatch):
    rng = np.random.default_rng(10)
    L, d = 50, 8
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    full = A.attn_fwd_dense(Q, K, V, 0.3) + A.attn_bwd_dense(Q, K, V, dO, 0.3)
    monkeypatch.setattr(A, "_ROW_BLOCK_BYTES", 8 * L * 7)   # 7 rows at a time
    blocked = A.attn_fwd_dense(Q, K, V, 0.3) + A.attn_bwd_dense(Q, K, V, dO, 0.3)
    for a, b in zip(full, blocked):
        assert np.max(np.abs(a - b)) <= 1e-12


def test_sampled_rows_and_columns_equal_full_evaluation():
    rng = np.random.default_rng(11)
    L, d = 45, 8
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    O, LSE = A.attn_fwd_dense(Q, K, V, 0.3)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, 0.3)
    rows = [0, 7, 44, 13]
    o_r, lse_r, dq_r = A.attn_query_rows(Q, K, V, dO, rows, 0.3)
    assert np.max(np.abs(o_r - O[rows])) <= 1e-13
    assert np.max(np.abs(lse_r - LSE[rows])) <= 1e-13
    assert np.max(np.abs(dq_r - dQ[rows])) <= 1e-12
    cols = [44, 2, 19]
    dk_c, dv_c = A.attn_key_cols(Q, K, V, dO, cols, 0.3)
    assert np.max(np.abs(dk_c - dK[cols])) <= 1e-12
    assert np.max(np.abs(dv_c - dV[cols])) <= 1e-12


# ----------------------------------------------------------------- planted mistakes (CPU only)

@pytest.mark.parametrize("mutation", ["drop_scale_dq", "sign_ds", "transpose_dk", "lse_without_max"])
def test_pins_catch_planted_mistakes(mutation):
    """Each planted mistake in a copy of the backward/forward formulas must break a pin above."""
    rng = np.random.default_rng(12)
    L, d = 12, 4
    Q, K, V, dO = (_rand(rng, L, d) for _ in range(4))
    scale = 0.7
    S = scale * Q @ K.T
    P, lse = A.softmax_rows(S)
    dP = dO @ V.T
    D = (P * dP).sum(axis=1, keepdims=True)
    dS = P * (dP - D)
    dQ, dK, dV = A.attn_bwd_dense(Q, K, V, dO, scale)
    if mutation == "drop_scale_dq":
        bad = dS @ K
        assert abs((Q * bad).sum() - (K * dK).sum()) > 1e-6      # <Q,dQ> = <K,dK> fails
    elif mutation == "sign_ds":
        bad = scale * (P * (D - dP)) @ K
        assert np.linalg.norm(bad - dQ) / np.linalg.norm(dQ) > 1.0
    elif mutation == "transpose_dk":
        bad = scale * dS @ Q                                     # dS instead of dS^T
        assert np.linalg.norm(bad - dK) / np.linalg.norm(dK) > 1e-3
    else:
        bad = np.log(np.exp(S).sum(axis=1)) + 1.0                # an offset LSE
        assert np.max(np.abs(np.exp(S - bad[:, None]).sum(axis=1) - 1.0)) > 0.1
