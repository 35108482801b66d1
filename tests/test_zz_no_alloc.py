"""knap_varlen_attn_bwd_noalloc (the backward whose scratch lives in the library's device image, for
callers that cannot allocate) against knap_varlen_attn_bwd with a caller workspace: same kernels, so the
results must agree bit for bit, which is within every bar the workspace variant is held to against the
oracle.  Two calls in a row, the second on a smaller bag (the scratch keeps the first call's contents)."""
import numpy as np
import pytest

import paper_2508_06001_amd as K
from knap_inputs import BagSpec, cu_seqlens_of, make_qkv_dout

from gpu_util import say


def test_scratch_limit_is_checked_before_anything_else_on_the_host():
    f = K.lib.knap_varlen_attn_bwd_noalloc
    big_T = K.KNAP_NOALLOC_MAX_ROWS // 24 + 1
    assert f(256, 512, 768, 1024, 1, 24, 128, 0.1, 1280, 1536, 1792, 2048, 2304, 2560, big_T, 0) \
        == K.KNAP_ERR_SCRATCH_TOO_SMALL
    assert f(0, 0, 0, 0, 0, 2, 64, 0.125, 0, 0, 0, 0, 0, 0, 0, 0) == K.KNAP_OK          # empty bag
    assert f(0, 0, 0, 0, 1, 2, 64, 0.125, 0, 0, 0, 0, 0, 0, 10, 0) == K.KNAP_ERR_INVALID_ARG   # null pointers
    assert "scratch" in K.knap_strerror(K.KNAP_ERR_SCRATCH_TOO_SMALL)


@pytest.mark.gpu
def test_noalloc_backward_equals_workspace_backward_twice_in_a_row():
    import torch
    from paper_2508_06001_amd.runtime import bf16_bits_to_device
    rng = np.random.default_rng(77)
    bags = [BagSpec("noalloc_first", [int(x) for x in rng.integers(50, 2600, size=12)] + [0, 1], H=6, d=128, seed=8801),
            BagSpec("noalloc_second_smaller", [700, 65, 129, 300], H=2, d=64, seed=8802)]
    for bag in bags:
        say(f"[gpu] noalloc bag={bag.name} T={bag.total_tokens} H={bag.H} d={bag.d}")
        bits = make_qkv_dout(bag)
        dev = {n: bf16_bits_to_device(bits[n]) for n in bits}
        cu = cu_seqlens_of(bag.seq_lens)
        attn = K.VarlenAttention(cu, bag.H, bag.d, bag.scale)
        attn.forward(dev["q"], dev["k"], dev["v"])
        dq, dk, dv = (t.clone() for t in attn.backward(dev["q"], dev["k"], dev["v"], dev["dout"]))
        torch.cuda.synchronize()
        T, H, d = bag.total_tokens, bag.H, bag.d
        g = 64                                             # NaN guard rows around each output
        big = [torch.full((T + 2 * g, H, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        out2 = [b[g:g + T] for b in big]
        rc = K.knap_varlen_attn_bwd_noalloc(dev["q"], dev["k"], dev["v"], attn.cu, attn.n_seq, H, d, bag.scale,
                                            attn.out, attn.lse, dev["dout"], out2[0], out2[1], out2[2], T)
        assert rc == K.KNAP_OK
        torch.cuda.synchronize()
        for name, want, got, b in zip(("dq", "dk", "dv"), (dq, dk, dv), out2, big):
            assert torch.equal(want.view(torch.int16), got.view(torch.int16)), (bag.name, name)
            assert bool(torch.isnan(b[:g]).all()) and bool(torch.isnan(b[g + T:]).all()), (bag.name, name)
    # a bag past the limit is refused and enqueues nothing
    too_many = K.KNAP_NOALLOC_MAX_ROWS // 2 + 1
    rc = K.knap_varlen_attn_bwd_noalloc(dev["q"], dev["k"], dev["v"], attn.cu, 1, 2, 64, 0.125, attn.out, attn.lse,
                                        dev["dout"], out2[0], out2[1], out2[2], too_many, check=False)
    assert rc == K.KNAP_ERR_SCRATCH_TOO_SMALL
