"""CPU oracle for the local (one-GPU) data movement of the Ulysses layout switch.

TEST INFRASTRUCTURE ONLY: imported by the tests and by the benchmark's
cpu_baseline leg, never by the library, and sharing no code with the HIP path.

What it computes.  Sec. 3.4 switches a multi-GPU bag between two layouts,
(partial sequences, full heads) and (full sequences, partial heads), with one
all-to-all before attention and one after it.  Sec. 3.3 (second pass) fixes the
first layout: a sequence of length L assigned to a g-GPU bag is cut into g
contiguous chunks as even as possible, chunk r going to GPU r of the bag;
every GPU packs its chunks in the bag's sequence order.  An all-to-all sends
contiguous buffers, so around it every GPU of the bag has to

  before sending   pack_heads      (T_r, H, d)  ->  g slabs (T_r, H/g, d), slab r' = heads of GPU r'
  after receiving  gather_chunks   g slabs (T_r, H/g, d), one per source GPU r
                                   ->  (T, H/g, d): every sequence whole, chunks in order r = 0..g-1

and the inverse of each on the way back (scatter_chunks, then unpack_heads).
These are pure permutations of (token, head) rows, so the oracle is the
definition written as plain slicing and Python loops over (sequence, GPU).

READING (the text says "evenly partition"): the first L mod g chunks are one
token longer.  T_r = sum_s c(s, r), T = sum_s L_s.

Pins (tests/test_oracle_ulysses.py): the defining property of the switch on a
simulated bag (what GPU r' ends with is exactly its heads of the unsplit
tensor), inverses, element-by-element brute force, and the row map being a
bijection that keeps each chunk contiguous.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def chunk_lengths(L: int, g: int) -> List[int]:
    """Lengths of the g contiguous chunks of one sequence (Sec. 3.3, second pass)."""
    base, rem = divmod(int(L), int(g))
    return [base + (1 if r < rem else 0) for r in range(g)]


def local_tokens(seq_lens: Sequence[int], g: int, r: int) -> int:
    """T_r: tokens GPU r of the bag holds in the (partial sequences, full heads) layout."""
    return sum(chunk_lengths(L, g)[r] for L in seq_lens)


def split_to_ranks(x: np.ndarray, seq_lens: Sequence[int], g: int) -> List[np.ndarray]:
    """The (partial sequences, full heads) layout of a packed tensor x (T, ...): what each GPU holds."""
    parts: List[List[np.ndarray]] = [[] for _ in range(g)]
    row = 0
    for L in seq_lens:
        for r, c in enumerate(chunk_lengths(L, g)):
            parts[r].append(x[row:row + c])
            row += c
    return [np.concatenate(p, axis=0) if p else x[:0] for p in parts]


def pack_heads(x: np.ndarray, g: int) -> np.ndarray:
    """(T_r, H, d) -> (g, T_r, H/g, d): slab r' holds heads [r' H/g, (r'+1) H/g) of every local token."""
    T, H, d = x.shape
    assert H % g == 0
    hg = H // g
    y = np.empty((g, T, hg, d), dtype=x.dtype)
    for rp in range(g):
        y[rp] = x[:, rp * hg:(rp + 1) * hg, :]
    return y


def unpack_heads(y: np.ndarray) -> np.ndarray:
    """Inverse of pack_heads: (g, T_r, H/g, d) -> (T_r, H, d)."""
    g, T, hg, d = y.shape
    x = np.empty((T, g * hg, d), dtype=y.dtype)
    for rp in range(g):
        x[:, rp * hg:(rp + 1) * hg, :] = y[rp]
    return x


def gather_chunks(slabs: Sequence[np.ndarray], seq_lens: Sequence[int]) -> np.ndarray:
    """Received slabs (one per source GPU r, each (T_r, H/g, d), chunks in sequence order) -> the
    (full sequences, partial heads) tensor (T, H/g, d)."""
    g = len(slabs)
    out = []
    taken = [0] * g
    for L in seq_lens:
        for r, c in enumerate(chunk_lengths(L, g)):
            out.append(slabs[r][taken[r]:taken[r] + c])
            taken[r] += c
    assert all(taken[r] == slabs[r].shape[0] for r in range(g))
    return np.concatenate(out, axis=0) if out else slabs[0][:0]


def scatter_chunks(z: np.ndarray, seq_lens: Sequence[int], g: int) -> List[np.ndarray]:
    """Inverse of gather_chunks: (T, H/g, d) -> g slabs, slab r = chunk r of every sequence."""
    return split_to_ranks(z, seq_lens, g)


def row_map(seq_lens: Sequence[int], g: int) -> np.ndarray:
    """For every row t of the (full sequences) tensor, its row in the concatenation of the g received
    slabs (slab 0 first): gather is z[t] = recv[row_map[t]], scatter is send[row_map[t]] = z[t]."""
    T_r = [local_tokens(seq_lens, g, r) for r in range(g)]
    slab_start = np.concatenate([[0], np.cumsum(T_r)])[:g]
    taken = [0] * g
    m = []
    for L in seq_lens:
        for r, c in enumerate(chunk_lengths(L, g)):
            m.extend(range(int(slab_start[r]) + taken[r], int(slab_start[r]) + taken[r] + c))
            taken[r] += c
    return np.asarray(m, dtype=np.int64)
