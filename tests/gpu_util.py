"""Helpers for the GPU parity tests: run the HIP path on seeded inputs and bring
the results back as float64 numpy arrays.  No oracle input or expected value is
ever taken from here."""
from __future__ import annotations

import sys

import numpy as np

from knap_inputs import BagSpec, bf16_bits_to_f32, cu_seqlens_of, make_qkv_dout


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


GUARD_ROWS = 64     # NaN rows in front of and behind every output tensor


class GuardedOutputs:
    """Replaces the output tensors of a VarlenAttention by views into larger allocations that start as
    NaN everywhere.  After a call the guard bands on both sides must still be NaN (nothing was written
    before row 0 or from row T on) and every element in between must be finite (nothing was left
    unwritten: NaN is the canary)."""

    def __init__(self, attn, backward: bool):
        import torch
        self.attn = attn
        T, H, d = attn.T, attn.H, attn.d
        self.big = {}
        names = ["out"] + (["dq", "dk", "dv"] if backward else [])
        if backward:
            attn._ensure_bwd_buffers()
        for n in names:
            big = torch.full((T + 2 * GUARD_ROWS, H, d), float("nan"), dtype=torch.bfloat16, device=attn.device)
            self.big[n] = big
            setattr(attn, n, big[GUARD_ROWS:GUARD_ROWS + T])
        g = GUARD_ROWS * 4
        big = torch.full((H * T + 2 * g,), float("nan"), dtype=torch.float32, device=attn.device)
        self.big["lse"] = big
        attn.lse = big[g:g + H * T].view(H, T)
        self.lse_guard = g

    def check(self, names) -> None:
        import torch
        for n in names:
            big = self.big[n]
            g = self.lse_guard if n == "lse" else GUARD_ROWS
            assert bool(torch.isnan(big[:g]).all()), f"{n}: written in front of the tensor"
            assert bool(torch.isnan(big[big.shape[0] - g:]).all()), f"{n}: written past the end of the tensor"
            assert bool(torch.isfinite(big[g:big.shape[0] - g]).all()), f"{n}: an element was left unwritten or is not finite"


class GpuRun:
    """q, k, v, dout on the device, one forward and one backward through the C ABI.  Every output
    tensor sits between NaN guard bands and starts as NaN; the run asserts that the bands are intact
    and that the whole of every output is finite, whatever the test then samples."""

    def __init__(self, bag: BagSpec, tensors=None, backward: bool = True, causal: bool = False, device_tensors=None):
        import torch
        import paper_2508_06001_amd as K
        from paper_2508_06001_amd.runtime import bf16_bits_to_device, bf16_device_to_bits

        self.bag = bag
        self.cu = cu_seqlens_of(bag.seq_lens)
        say(f"[gpu] bag={bag.name} seed={bag.seed} n_seq={len(bag.seq_lens)} T={bag.total_tokens} "
            f"H={bag.H} d={bag.d} maxL={max(bag.seq_lens) if bag.seq_lens else 0} causal={causal}")
        if device_tensors is not None:        # inputs made on the device (closed-form cases): no host copy kept
            self.bits = None
            dev = device_tensors
        else:
            self.bits = tensors if tensors is not None else make_qkv_dout(bag)
            dev = {n: bf16_bits_to_device(self.bits[n]) for n in ("q", "k", "v", "dout")}
        self.dev = dev
        self.attn = K.VarlenAttention(self.cu, bag.H, bag.d, bag.scale, causal=causal)
        self.guards = GuardedOutputs(self.attn, backward)
        say("[gpu] forward")
        self.attn.forward(dev["q"], dev["k"], dev["v"])
        torch.cuda.synchronize()
        self.guards.check(["out", "lse"])
        if device_tensors is None:
            self.out_bits = bf16_device_to_bits(self.attn.out)
            self.lse = self.attn.lse.cpu().numpy().astype(np.float64)
        if backward:
            say("[gpu] backward")
            self.attn.backward(dev["q"], dev["k"], dev["v"], dev["dout"])
            torch.cuda.synchronize()
            self.guards.check(["out", "lse", "dq", "dk", "dv"])
            if device_tensors is None:
                self.dq_bits = bf16_device_to_bits(self.attn.dq)
                self.dk_bits = bf16_device_to_bits(self.attn.dk)
                self.dv_bits = bf16_device_to_bits(self.attn.dv)
        say("[gpu] done")

    def host(self, name: str, rows: slice, head: int) -> np.ndarray:
        """float64 view of rows of one head of an input or output tensor."""
        src = {"out": getattr(self, "out_bits", None), "dq": getattr(self, "dq_bits", None),
               "dk": getattr(self, "dk_bits", None), "dv": getattr(self, "dv_bits", None)}.get(name)
        if src is None:
            src = self.bits[name]
        return to_f64(src[rows, head, :])


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    nb = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (nb if nb > 0 else 1.0)
