"""The causal zero-score closed forms used at full size on the GPU, checked here against the oracle's causal
mode on sequences small enough for its L x L pass (both blockings of the carried sums: several blocks with a
ragged last one, and a single block)."""
import numpy as np
import pytest

from oracle import attention as A

from causal_closed_forms import causal_zero_score_reference


@pytest.mark.parametrize("zero", ["k", "q"])
@pytest.mark.parametrize("L,block", [(301, 64), (97, 1024), (1, 8)])
def test_zero_score_closed_form_equals_oracle(zero, L, block):
    import torch
    rng = np.random.default_rng(1000 + L)
    H, d, scale = 2, 16, 0.37
    x = {n: rng.standard_normal((L, H, d)) for n in ("q", "k", "v", "do")}
    x[zero] = np.zeros((L, H, d))
    t = {n: torch.from_numpy(a) for n, a in x.items()}
    out, lse, dq, dk, dv = causal_zero_score_reference(t["q"], t["k"], t["v"], t["do"], scale, block=block)
    for h in range(H):
        Q, K_, V, dO = (x[n][:, h, :] for n in ("q", "k", "v", "do"))
        O, LSE = A.attn_fwd_dense(Q, K_, V, scale, causal=True)
        dQ, dK, dV = A.attn_bwd_dense(Q, K_, V, dO, scale, causal=True)
        np.testing.assert_allclose(out[:, h, :].numpy(), O, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[h].numpy(), LSE, rtol=0, atol=1e-12)
        np.testing.assert_allclose(dv[:, h, :].numpy(), dV, rtol=0, atol=1e-12)
        np.testing.assert_allclose(dq[:, h, :].numpy(), dQ, rtol=0, atol=1e-11)
        np.testing.assert_allclose(dk[:, h, :].numpy(), dK, rtol=0, atol=1e-11)
    if zero == "k":
        assert float(dq.abs().max()) == 0.0
    else:
        assert float(dk.abs().max()) == 0.0
