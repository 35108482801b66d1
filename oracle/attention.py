"""CPU oracle for packed variable-length joint self-attention, forward and backward.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP
kernels are compared against.  It is imported by the tests, by the smoke check
and by the benchmark's cpu_baseline leg, never by the library itself, and it
shares no code with the HIP path.

What it computes (Sec. 3.4 and the attention listing of Sec. 3.5: packed q, k, v
of shape (l1+...+ln, h, d) attended per sequence as delimited by seq_lens;
Limitations paragraph: bidirectional full attention inside each datum; Eq. 1:
the attention term is exactly two l x l x d contractions per head).  FlashAttention
is an exact reformulation of softmax attention, so the oracle is the plain
definition, evaluated in float64 for every (sequence, head) independently:

    S   = scale * Q K^T                       (L x L)
    P   = softmax over each row of S          LSE_i = log sum_j exp(S_ij)
    O   = P V
    dV  = P^T dO
    dP  = dO V^T
    D_i = sum_j P_ij dP_ij                    (equals sum_c dO_ic O_ic)
    dS  = P * (dP - D)                        (row-wise D)
    dQ  = scale * dS K
    dK  = scale * dS^T Q

The other homogeneous mask the paper admits inside a datum (Limitations
paragraph: bidirectional full attention or causal attention) is the same
definition with S_ij = -inf for j > i, i and j counted from the start of the
sequence: ``causal=True``.  A masked score has P_ij = 0 and takes no part in any
sum; row i then depends on keys 0..i only.

Matrix products use numpy's matmul (a library primitive per step).  Long
sequences are evaluated a block of query rows at a time only to bound memory:
every row still sees its whole row of scores, there is no online softmax.

Parity pins (tests/test_oracle_attention.py): scalar-loop brute force over the
packed T x T masked problem, closed forms (constant V, zero K, L = 1, one-hot
limit), central finite differences, torch float64 autograd on a single
sequence, and algebraic invariants of the backward.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

_ROW_BLOCK_BYTES = 256 << 20  # bound for one L-wide block of fp64 scores


def _row_block(L: int) -> int:
    return max(1, min(L, _ROW_BLOCK_BYTES // (8 * max(L, 1))))


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def softmax_rows(S: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Row softmax of a score block and the row log-sum-exp."""
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    return E / l, (m + np.log(l))[:, 0]


def _mask_future_keys(S: np.ndarray, rows: np.ndarray) -> None:
    """Causal mask, in place: score (i, j) of query row rows[i] is -inf where j > rows[i]."""
    S[np.arange(S.shape[1])[None, :] > np.asarray(rows)[:, None]] = -np.inf


def attn_fwd_dense(Q, K, V, scale: float, causal: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """One sequence, one head.  Q, K, V: (L, d).  Returns O (L, d) and LSE (L,)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L = Q.shape[0]
    O = np.empty_like(Q)
    LSE = np.empty(L, dtype=np.float64)
    rb = _row_block(L)
    for r0 in range(0, L, rb):
        r1 = min(L, r0 + rb)
        S = scale * (Q[r0:r1] @ K.T)
        if causal:
            _mask_future_keys(S, np.arange(r0, r1))
        P, lse = softmax_rows(S)
        O[r0:r1] = P @ V
        LSE[r0:r1] = lse
    return O, LSE


def attn_bwd_dense(Q, K, V, dO, scale: float, causal: bool = False) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One sequence, one head.  Gradients of sum(dO * O) with respect to Q, K, V."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    L = Q.shape[0]
    dQ = np.empty_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    rb = _row_block(L)
    for r0 in range(0, L, rb):
        r1 = min(L, r0 + rb)
        S = scale * (Q[r0:r1] @ K.T)
        if causal:
            _mask_future_keys(S, np.arange(r0, r1))
        P, _ = softmax_rows(S)
        dV += P.T @ dO[r0:r1]
        dP = dO[r0:r1] @ V.T
        D = (P * dP).sum(axis=1, keepdims=True)
        dS = P * (dP - D)
        dQ[r0:r1] = scale * (dS @ K)
        dK += scale * (dS.T @ Q[r0:r1])
    return dQ, dK, dV


def varlen_attn_fwd(q, k, v, cu_seqlens: Sequence[int], scale: float,
                    causal: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Packed forward.  q, k, v: (T, H, d).  Returns out (T, H, d) and lse (H, T), float64.

    Each sequence is sliced out and attended on its own; nothing is ever formed
    across sequences.  Zero-length sequences are skipped.
    """
    T, H, d = np.shape(q)
    out = np.zeros((T, H, d), dtype=np.float64)
    lse = np.zeros((H, T), dtype=np.float64)
    cu = [int(c) for c in cu_seqlens]
    for s in range(len(cu) - 1):
        r0, r1 = cu[s], cu[s + 1]
        if r1 <= r0:
            continue
        for h in range(H):
            O, LSE = attn_fwd_dense(q[r0:r1, h, :], k[r0:r1, h, :], v[r0:r1, h, :], scale, causal)
            out[r0:r1, h, :] = O
            lse[h, r0:r1] = LSE
    return out, lse


def varlen_attn_bwd(q, k, v, cu_seqlens: Sequence[int], scale: float, dout, causal: bool = False):
    """Packed backward.  Returns dq, dk, dv, each (T, H, d) float64."""
    T, H, d = np.shape(q)
    dq = np.zeros((T, H, d), dtype=np.float64)
    dk = np.zeros((T, H, d), dtype=np.float64)
    dv = np.zeros((T, H, d), dtype=np.float64)
    cu = [int(c) for c in cu_seqlens]
    for s in range(len(cu) - 1):
        r0, r1 = cu[s], cu[s + 1]
        if r1 <= r0:
            continue
        for h in range(H):
            dQ, dK, dV = attn_bwd_dense(q[r0:r1, h, :], k[r0:r1, h, :], v[r0:r1, h, :],
                                        dout[r0:r1, h, :], scale, causal)
            dq[r0:r1, h, :] = dQ
            dk[r0:r1, h, :] = dK
            dv[r0:r1, h, :] = dV
    return dq, dk, dv


# ---------------------------------------------------------------------------
# Exact evaluation of selected outputs of one long (sequence, head)
# ---------------------------------------------------------------------------

def attn_query_rows(Q, K, V, dO, rows: Sequence[int], scale: float, causal: bool = False):
    """Exact O, LSE and dQ for the chosen query rows of one (sequence, head).

    A query row depends only on its own q and dO rows and on all of K and V, so
    these are the same formulas as above restricted to the chosen rows.
    Q, dO may be the full (L, d) arrays; only ``rows`` of them are read.
    """
    rows = np.asarray(rows, dtype=np.int64)
    K, V = _f64(K), _f64(V)
    Qr = _f64(np.asarray(Q)[rows])
    dOr = _f64(np.asarray(dO)[rows])
    S = scale * (Qr @ K.T)
    if causal:
        _mask_future_keys(S, rows)
    P, lse = softmax_rows(S)
    O = P @ V
    dP = dOr @ V.T
    D = (P * dP).sum(axis=1, keepdims=True)
    dS = P * (dP - D)
    dQ = scale * (dS @ K)
    return O, lse, dQ


def attn_key_cols(Q, K, V, dO, cols: Sequence[int], scale: float, causal: bool = False):
    """Exact dK and dV for the chosen key/value rows of one (sequence, head).

    Needs LSE_i and D_i of every query row, so one full forward pass over the
    sequence is made first (in row blocks); then only the chosen columns of P,
    dP and dS are formed.
    """
    cols = np.asarray(cols, dtype=np.int64)
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    O, LSE = attn_fwd_dense(Q, K, V, scale, causal)
    D = (dO * O).sum(axis=1)
    Kc, Vc = K[cols], V[cols]
    Sc = scale * (Q @ Kc.T)                 # (L, n_cols)
    if causal:                              # key cols[c] is in the future of query i when cols[c] > i
        Sc[cols[None, :] > np.arange(Q.shape[0])[:, None]] = -np.inf
    Pc = np.exp(Sc - LSE[:, None])
    dPc = dO @ Vc.T
    dSc = Pc * (dPc - D[:, None])
    dVc = Pc.T @ dO
    dKc = scale * (dSc.T @ Q)
    return dKc, dVc
