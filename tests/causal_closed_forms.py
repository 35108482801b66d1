"""Closed form of causal attention when every visible score is zero (K = 0 or Q = 0), written out from the
definition (Sec. 3.4 with the mask "query i sees keys 0..i"; Eq. 1): P_ij = 1 / (i + 1) for j <= i.

    O_i   = (V_0 + ... + V_i) / (i + 1)                  LSE_i = ln(i + 1)
    dV_j  = sum_{i >= j} g_i,   g_i = dO_i / (i + 1)
    dS_ij = (dO_i . (V_j - O_i)) / (i + 1)
    dQ_i  = scale sum_{j <= i} dS_ij K_j = scale (C_i g_i - w_i ksum_i)
            with C_i = sum_{j <= i} K_j V_j^T, ksum_i = sum_{j <= i} K_j, w_i = (dO_i . O_i) / (i + 1)
    dK_j  = scale sum_{i >= j} dS_ij Q_i = scale (A_j V_j - b_j)
            with A_j = sum_{i >= j} Q_i g_i^T, b_j = sum_{i >= j} w_i Q_i

The d x d prefix and suffix sums C_i and A_j are carried from block to block of rows (the pairs inside a block
are summed directly), which makes the cost O(L d^2 + L B d) per head instead of O(L^2 d).  Nothing here calls
the library or the oracle: the CPU suite checks these formulas against the oracle's causal mode on a small
sequence, the GPU suite checks the library against them at full size."""


def causal_zero_score_reference(q, k, v, do, scale: float, block: int = 1024):
    """q, k, v, do: float64 torch tensors (L, H, d) of ONE sequence, with q = 0 or k = 0.
    Returns out (L, H, d), lse (H, L), dq, dk, dv (L, H, d), float64, on the tensors' device."""
    import torch
    L, H, d = v.shape
    n = torch.arange(1, L + 1, dtype=torch.float64, device=v.device).view(L, 1, 1)
    out = torch.cumsum(v, dim=0) / n
    lse = torch.log(n.view(1, L)).expand(H, L)
    g = do / n
    dv = torch.flip(torch.cumsum(torch.flip(g, dims=[0]), dim=0), dims=[0])
    w = (do * out).sum(dim=-1, keepdim=True) / n                      # (L, H, 1)
    ksum = torch.cumsum(k, dim=0)
    b = torch.flip(torch.cumsum(torch.flip(q * w, dims=[0]), dim=0), dims=[0])
    dq = torch.empty_like(v)
    dk = torch.empty_like(v)
    # forward sweep: C = sum of K_j V_j^T over the rows before the block
    C = torch.zeros((H, d, d), dtype=torch.float64, device=v.device)
    for j0 in range(0, L, block):
        j1 = min(L, j0 + block)
        m = torch.einsum("ihe,jhe->hij", g[j0:j1], v[j0:j1])         # m[h, i, j] = g_i . V_j
        m = torch.tril(m)                                             # j <= i
        inside = torch.einsum("hij,jhc->ihc", m, k[j0:j1])
        before = torch.einsum("hce,ihe->ihc", C, g[j0:j1])
        dq[j0:j1] = scale * (inside + before - w[j0:j1] * ksum[j0:j1])
        C += torch.einsum("jhc,jhe->hce", k[j0:j1], v[j0:j1])
    # backward sweep: A = sum of Q_i g_i^T over the rows after the block
    A = torch.zeros((H, d, d), dtype=torch.float64, device=v.device)
    starts = list(range(0, L, block))
    for j0 in reversed(starts):
        j1 = min(L, j0 + block)
        m = torch.einsum("ihe,jhe->hij", g[j0:j1], v[j0:j1])
        m = torch.tril(m)                                             # i >= j
        inside = torch.einsum("hij,ihc->jhc", m, q[j0:j1])
        after = torch.einsum("hce,jhe->jhc", A, v[j0:j1])
        dk[j0:j1] = scale * (inside + after - b[j0:j1])
        A += torch.einsum("ihc,ihe->hce", q[j0:j1], g[j0:j1])
    return out, lse, dq, dk, dv
