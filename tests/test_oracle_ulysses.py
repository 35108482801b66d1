"""Pins of the Ulysses data-movement oracle against things other than itself.

* the defining property of the layout switch (Sec. 3.4): simulate a whole g-GPU bag on the host
  -- split a packed (T, H, d) tensor into per-GPU chunks (Sec. 3.3, second pass), pack, exchange slab
  r' of GPU r with slab r of GPU r' (the all-to-all, done here by list indexing), gather -- and GPU
  r' must hold exactly heads [r' H/g, (r'+1) H/g) of the unsplit tensor;
* the way back restores every GPU's input;
* element-by-element brute force of both permutations on a tiny case;
* the row map is a bijection, keeps chunks contiguous and ordered, and reproduces gather / scatter;
* chunk lengths: sum to L, differ by at most one, longer ones first;
* planted mistakes (interleaved instead of contiguous head blocks, chunks left in GPU-major order) break
  the property.  (Any chunk rule used consistently satisfies the property; the rule itself is the stated
  reading, pinned by test_chunk_lengths and by the explicit rows of the brute-force case.)
"""
import numpy as np
import pytest

from oracle import ulysses as U


def _bag(rng, seq_lens, H, d):
    T = int(sum(seq_lens))
    # distinct integers: any misplaced element is visible
    return np.arange(T * H * d, dtype=np.int64).reshape(T, H, d) * 3 + rng.integers(0, 3, size=(T, H, d))


def _simulate_switch(x, seq_lens, g):
    local = U.split_to_ranks(x, seq_lens, g)                    # (partial sequences, full heads)
    sent = [U.pack_heads(xr, g) for xr in local]                # sent[r][r'] goes from GPU r to GPU r'
    received = [[sent[r][rp] for r in range(g)] for rp in range(g)]
    return local, [U.gather_chunks(received[rp], seq_lens) for rp in range(g)]


@pytest.mark.parametrize("g,H", [(2, 4), (4, 8), (8, 24), (3, 6), (8, 8)])
def test_switch_gives_every_gpu_its_heads_of_the_whole_sequences(g, H):
    rng = np.random.default_rng(100 + g)
    seq_lens = [17, 1, 0, 8, 5, 64, g - 1, g, g + 1, 3]          # shorter than g: some chunks are empty
    x = _bag(rng, seq_lens, H, 4)
    hg = H // g
    _, full = _simulate_switch(x, seq_lens, g)
    for rp in range(g):
        assert np.array_equal(full[rp], x[:, rp * hg:(rp + 1) * hg, :])


def test_way_back_restores_every_gpus_input():
    rng = np.random.default_rng(7)
    g, H, d = 4, 8, 2
    seq_lens = [9, 2, 31, 4]
    x = _bag(rng, seq_lens, H, d)
    local, full = _simulate_switch(x, seq_lens, g)
    back_sent = [U.scatter_chunks(full[rp], seq_lens, g) for rp in range(g)]   # back_sent[r'][r] returns to GPU r
    for r in range(g):
        y = np.stack([back_sent[rp][r] for rp in range(g)], axis=0)            # (g, T_r, H/g, d)
        assert np.array_equal(U.unpack_heads(y), local[r])
        assert np.array_equal(U.unpack_heads(U.pack_heads(local[r], g)), local[r])


def test_brute_force_tiny():
    g, H, d = 2, 4, 3
    seq_lens = [3, 2]
    T = 5
    x = np.arange(T * H * d).reshape(T, H, d)
    # pack_heads, element by element
    y = U.pack_heads(x, g)
    for rp in range(g):
        for t in range(T):
            for hl in range(H // g):
                for c in range(d):
                    assert y[rp, t, hl, c] == x[t, rp * (H // g) + hl, c]
    # chunks of [3, 2] on 2 GPUs: GPU 0 holds rows 0,1 (seq 0) and 3 (seq 1); GPU 1 holds row 2 and row 4
    local = U.split_to_ranks(x, seq_lens, g)
    assert np.array_equal(local[0], x[[0, 1, 3]]) and np.array_equal(local[1], x[[2, 4]])
    assert list(U.row_map(seq_lens, g)) == [0, 1, 3, 2, 4]       # receive buffer: GPU 0's 3 rows, then GPU 1's 2


@pytest.mark.parametrize("g", [1, 2, 5, 8])
def test_row_map_is_a_bijection_that_reproduces_gather_and_scatter(g):
    rng = np.random.default_rng(11 + g)
    seq_lens = [int(v) for v in rng.integers(0, 40, size=12)]
    T = sum(seq_lens)
    m = U.row_map(seq_lens, g)
    assert sorted(m.tolist()) == list(range(T))
    z = rng.standard_normal((T, 2, 3))
    slabs = U.scatter_chunks(z, seq_lens, g)
    recv = np.concatenate(slabs, axis=0)
    assert np.array_equal(recv[m], z)                            # gather
    send = np.empty_like(z)
    send[m] = z                                                  # scatter
    assert np.array_equal(send, recv)
    assert np.array_equal(U.gather_chunks(slabs, seq_lens), z)
    # inside one sequence the map is piecewise contiguous with at most g pieces, source GPUs ascending
    row = 0
    for L in seq_lens:
        seg = m[row:row + L]
        breaks = int(np.sum(np.diff(seg) != 1)) if L > 1 else 0
        assert breaks <= g - 1
        row += L


def test_chunk_lengths():
    for L in range(0, 70):
        for g in (1, 2, 3, 8):
            c = U.chunk_lengths(L, g)
            assert sum(c) == L and max(c) - min(c) <= 1 and c == sorted(c, reverse=True)
    assert U.chunk_lengths(10, 4) == [3, 3, 2, 2]


@pytest.mark.parametrize("mistake", ["interleaved_heads", "gpu_major_chunks"])
def test_property_catches_planted_mistakes(mistake):
    rng = np.random.default_rng(5)
    g, H, d = 2, 4, 2
    seq_lens = [5, 4]
    hg = H // g
    x = _bag(rng, seq_lens, H, d)
    local = U.split_to_ranks(x, seq_lens, g)
    if mistake == "interleaved_heads":
        # GPU r' given heads r', r' + g, ... instead of a contiguous block of H/g heads
        sent = [xr.reshape(-1, hg, g, d).transpose(2, 0, 1, 3) for xr in local]
        got = U.gather_chunks([sent[r][0] for r in range(g)], seq_lens)
    else:
        # the received slabs concatenated as they are: all of GPU 0's chunks, then all of GPU 1's
        sent = [U.pack_heads(xr, g) for xr in local]
        got = np.concatenate([sent[r][0] for r in range(g)], axis=0)
    assert not np.array_equal(got, x[:, :hg, :])
