"""Parity of the Ulysses data-movement kernels with the oracle: pure permutations, so bit-exact.

A whole g-GPU bag is simulated on the one GPU: every simulated rank's tensors go through the C ABI
(pack_heads, then -- after the all-to-all, which is done here by slicing on the host -- gather_chunks)
and back.  Checked against oracle/ulysses.py and against the defining property of the switch: rank r'
ends with exactly its heads of the unsplit packed tensor.
"""
import numpy as np
import pytest

from knap_inputs import cu_seqlens_of
from oracle import ulysses as U

from gpu_util import say

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def _host(t):
    return t.cpu().numpy().view(np.uint16)


def _plan(K, seq_lens, g):
    import torch
    cu = torch.from_numpy(np.asarray(cu_seqlens_of(seq_lens), dtype=np.int32)).cuda()
    T = int(sum(seq_lens))
    row_map = torch.full((max(T, 1),), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(K.knap_ulysses_plan_workspace_bytes(len(seq_lens), g), 256), dtype=torch.uint8, device="cuda")
    K.knap_ulysses_plan(cu, len(seq_lens), T, g, row_map, ws)
    torch.cuda.synchronize()
    return row_map


def _switch_and_back(seq_lens, g, H, d, seed):
    import torch
    import paper_2508_06001_amd as K
    say(f"[gpu] ulysses bag: n_seq={len(seq_lens)} T={sum(seq_lens)} g={g} H={H} d={d} seed={seed}")
    rng = np.random.default_rng(seed)
    T, hg = int(sum(seq_lens)), H // g
    x = rng.integers(0, 1 << 16, size=(T, H, d), dtype=np.uint16)        # bf16 bit patterns, any value
    local = U.split_to_ranks(x, seq_lens, g)
    T_r = [a.shape[0] for a in local]
    assert K.knap_ulysses_local_tokens(seq_lens, g) == T_r
    row_map = _plan(K, seq_lens, g)
    assert np.array_equal(row_map.cpu().numpy()[:T], U.row_map(seq_lens, g))
    # pack on every simulated rank
    sent = []
    for r in range(g):
        y = torch.full((g, T_r[r], hg, d), -1, dtype=torch.int16, device="cuda")
        K.knap_ulysses_pack_heads(_dev(local[r]), T_r[r], H, d, g, y)
        torch.cuda.synchronize()
        sent.append(_host(y))
        assert np.array_equal(sent[r], U.pack_heads(local[r], g)), ("pack", r)
    # all-to-all by slicing; gather on every rank
    full = []
    for rp in range(g):
        recv = np.concatenate([sent[r][rp] for r in range(g)], axis=0)
        z = torch.full((T, hg, d), -1, dtype=torch.int16, device="cuda")
        K.knap_ulysses_gather_chunks(_dev(recv), row_map, T, hg, d, z)
        torch.cuda.synchronize()
        full.append(_host(z))
        assert np.array_equal(full[rp], x[:, rp * hg:(rp + 1) * hg, :]), ("gather", rp)   # the defining property
        assert np.array_equal(full[rp], U.gather_chunks([sent[r][rp] for r in range(g)], seq_lens))
        # and straight back: scatter reproduces the receive buffer
        send = torch.full((T, hg, d), -1, dtype=torch.int16, device="cuda")
        K.knap_ulysses_scatter_chunks(z, row_map, T, hg, d, send)
        torch.cuda.synchronize()
        assert np.array_equal(_host(send), recv), ("scatter", rp)
    # second all-to-all by slicing; unpack on every rank restores its input
    for r in range(g):
        back = np.stack([U.scatter_chunks(full[rp], seq_lens, g)[r] for rp in range(g)], axis=0)
        xr = torch.full((T_r[r], H, d), -1, dtype=torch.int16, device="cuda")
        K.knap_ulysses_unpack_heads(_dev(back), T_r[r], H, d, g, xr)
        torch.cuda.synchronize()
        assert np.array_equal(_host(xr), local[r]), ("unpack", r)


@pytest.mark.parametrize("g,H,d", [(2, 4, 64), (4, 8, 128), (8, 24, 128), (3, 6, 64), (8, 8, 8), (1, 2, 64)])
def test_switch_and_back_on_ragged_bags(g, H, d):
    # lengths below, at and above g (empty chunks), zero-length sequences, lengths not divisible by g
    seq_lens = [1037, 1, 0, g - 1, g, g + 1, 513, 64, 0, 7, 300, 129]
    _switch_and_back(seq_lens, g, H, d, seed=600 + g)


def test_single_sequence_and_many_sequences():
    _switch_and_back([4099], 8, 16, 64, seed=71)
    rng = np.random.default_rng(72)
    _switch_and_back([int(v) for v in rng.integers(0, 60, size=2048)], 4, 4, 64, seed=73)   # KNAP_MAX_SEQS sequences


@pytest.mark.timeout(300)
def test_post_ulysses_share_at_full_size():
    """The 8-GPU bag behind benchmark config 4 (24 heads -> 3 per GPU, 196608 tokens): one rank's pack and
    one rank's gather at full size, every element compared."""
    import torch
    import paper_2508_06001_amd as K
    from knap_inputs import config_bag
    seq_lens = config_bag(4).seq_lens
    g, H, d = 8, 24, 128
    hg, T = H // g, sum(seq_lens)
    T_r = K.knap_ulysses_local_tokens(seq_lens, g)
    rng = np.random.default_rng(74)
    xr = rng.integers(0, 1 << 16, size=(T_r[3], H, d), dtype=np.uint16)
    y = torch.full((g, T_r[3], hg, d), -1, dtype=torch.int16, device="cuda")
    K.knap_ulysses_pack_heads(_dev(xr), T_r[3], H, d, g, y)
    torch.cuda.synchronize()
    assert np.array_equal(_host(y), U.pack_heads(xr, g))
    back = torch.full((T_r[3], H, d), -1, dtype=torch.int16, device="cuda")
    K.knap_ulysses_unpack_heads(y, T_r[3], H, d, g, back)
    torch.cuda.synchronize()
    assert np.array_equal(_host(back), xr)
    del y, back
    recv = rng.integers(0, 1 << 16, size=(T, hg, d), dtype=np.uint16)
    row_map = _plan(K, seq_lens, g)
    m = U.row_map(seq_lens, g)
    assert np.array_equal(row_map.cpu().numpy(), m)
    z = torch.full((T, hg, d), -1, dtype=torch.int16, device="cuda")
    K.knap_ulysses_gather_chunks(_dev(recv), row_map, T, hg, d, z)
    torch.cuda.synchronize()
    slabs = np.split(recv, np.cumsum(T_r)[:-1], axis=0)
    assert np.array_equal(_host(z), U.gather_chunks(slabs, seq_lens))
    send = torch.full((T, hg, d), -1, dtype=torch.int16, device="cuda")
    K.knap_ulysses_scatter_chunks(z, row_map, T, hg, d, send)
    torch.cuda.synchronize()
    assert np.array_equal(_host(send), recv)


@pytest.mark.timeout(300)
def test_multi_gpu_bag_end_to_end_on_one_gpu():
    """Sec. 3.4 end to end for a 4-GPU bag, every rank simulated on the one GPU: q, k, v start as
    (partial sequences, full heads); pack -> exchange -> gather -> packed attention on H/g heads ->
    scatter -> exchange -> unpack.  What every rank ends with must be its chunks of the attention of
    the whole sequences over all heads (fp64 oracle, the forward bars of the parity tests)."""
    import torch
    import paper_2508_06001_amd as K
    from knap_inputs import BagSpec, make_qkv_dout
    from oracle import attention as A
    from gpu_util import to_f64
    g, H, d = 4, 8, 128
    hg = H // g
    bag = BagSpec("ulysses_e2e", [700, 130, 3, 257, 1024], H=H, d=d, seed=881)
    seq_lens, T = bag.seq_lens, bag.total_tokens
    bits = make_qkv_dout(bag)                                    # the unsplit packed tensors
    cu = cu_seqlens_of(seq_lens)
    row_map = _plan(K, seq_lens, g)
    T_r = K.knap_ulysses_local_tokens(seq_lens, g)
    # every rank packs its q, k, v
    sent = {}
    for name in ("q", "k", "v"):
        local = U.split_to_ranks(bits[name], seq_lens, g)
        for r in range(g):
            y = torch.empty((g, T_r[r], hg, d), dtype=torch.int16, device="cuda")
            K.knap_ulysses_pack_heads(_dev(local[r]), T_r[r], H, d, g, y)
            torch.cuda.synchronize()
            sent[name, r] = _host(y)
    # every rank gathers whole sequences and attends with its H/g heads
    out_send = []
    for rp in range(g):
        full = {}
        for name in ("q", "k", "v"):
            recv = _dev(np.concatenate([sent[name, r][rp] for r in range(g)], axis=0))
            z = torch.empty((T, hg, d), dtype=torch.int16, device="cuda")
            K.knap_ulysses_gather_chunks(recv, row_map, T, hg, d, z)
            full[name] = z.view(torch.bfloat16)
        attn = K.VarlenAttention(cu, hg, d, bag.scale)
        attn.forward(full["q"], full["k"], full["v"])
        send = torch.empty((T, hg, d), dtype=torch.int16, device="cuda")
        K.knap_ulysses_scatter_chunks(attn.out.view(torch.int16), row_map, T, hg, d, send)
        torch.cuda.synchronize()
        out_send.append(np.split(_host(send), np.cumsum(T_r)[:-1], axis=0))     # slab r goes back to rank r
    # every rank unpacks; compare with the oracle on the unsplit problem
    f64 = {n: to_f64(bits[n]) for n in ("q", "k", "v")}
    o_ref, _ = A.varlen_attn_fwd(f64["q"], f64["k"], f64["v"], cu, bag.scale)
    ref_local = U.split_to_ranks(o_ref, seq_lens, g)
    for r in range(g):
        back = np.stack([out_send[rp][r] for rp in range(g)], axis=0)
        x = torch.empty((T_r[r], H, d), dtype=torch.int16, device="cuda")
        K.knap_ulysses_unpack_heads(_dev(back), T_r[r], H, d, g, x)
        torch.cuda.synchronize()
        err = np.abs(to_f64(_host(x)) - ref_local[r])
        err = np.where(err <= 2.0 ** -8 * np.abs(ref_local[r]), 0.0, err)       # bf16 resolution of the stored output
        say(f"[parity] ulysses end to end, rank {r}: max|err|={float(err.max()):.3e}")
        assert float(err.max()) <= 1e-2
