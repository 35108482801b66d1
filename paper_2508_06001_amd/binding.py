"""ctypes binding of libknapattn.so: the same names as include/knapattn.h (and the benchmark hooks of
include/knapattn_bench.h).

Argument marshalling only.  Every step of the attention path runs in the HIP
kernels of the shared library; PyTorch supplies device memory and the stream.
There is no fallback: if the library has not been built the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libknapattn.so")

KNAP_OK = 0
KNAP_ERR_INVALID_ARG = -1
KNAP_ERR_WORKSPACE_TOO_SMALL = -2
KNAP_ERR_LAUNCH_FAILED = -3
KNAP_ERR_TOO_MANY_SEQS = -4
KNAP_ERR_CAPACITY = -5
KNAP_ERR_PARSE = -6
KNAP_ERR_SCRATCH_TOO_SMALL = -7
KNAP_NOALLOC_MAX_ROWS = 4 * 1024 * 1024
KNAP_MAX_SEQS = 2048
KNAP_ULYSSES_MAX_GPUS = 64

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first with `python paper_2508_06001_amd/build.py` "
        "(there is no CPU or PyTorch fallback for the attention path)")

# PyTorch ships its own HIP runtime (same SONAME as the system one).  It must be
# in the process before this library is loaded, so that both resolve to ONE
# runtime: streams and device pointers handed over by PyTorch are only valid in
# the runtime that created them.
import torch  # noqa: E402,F401

lib = C.CDLL(LIB_PATH)

_vp, _i, _f, _d, _i64, _sz = C.c_void_p, C.c_int, C.c_float, C.c_double, C.c_int64, C.c_size_t
_pd, _pi, _pi64, _pi32 = C.POINTER(C.c_double), C.POINTER(C.c_int), C.POINTER(C.c_int64), C.POINTER(C.c_int32)

_SIGNATURES = {
    "knap_varlen_attn_fwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _f, _vp, _vp, _vp]),
    "knap_varlen_attn_bwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _f, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "knap_varlen_attn_bwd_workspace_bytes": (_sz, [_i64, _i, _i, _i]),
    "knap_varlen_attn_bwd_noalloc": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _f, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp]),
    "knap_varlen_attn_causal_fwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _f, _vp, _vp, _vp]),
    "knap_varlen_attn_causal_bwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _f, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "knap_ulysses_pack_heads": (_i, [_vp, _i64, _i, _i, _i, _vp, _vp]),
    "knap_ulysses_unpack_heads": (_i, [_vp, _i64, _i, _i, _i, _vp, _vp]),
    "knap_ulysses_plan_workspace_bytes": (_sz, [_i, _i]),
    "knap_ulysses_plan": (_i, [_vp, _i, _i64, _i, _vp, _vp, _sz, _vp]),
    "knap_ulysses_gather_chunks": (_i, [_vp, _vp, _i64, _i, _i, _vp, _vp]),
    "knap_ulysses_scatter_chunks": (_i, [_vp, _vp, _i64, _i, _i, _vp, _vp]),
    "knap_ulysses_local_tokens": (_i, [_pi64, _i, _i, _pi64]),
    "knap_strerror": (C.c_char_p, [_i]),
    "knap_last_hip_error": (_i, []),
    "knap_launch_workgroups": (_i, [_i]),
    "knap_bwd_profile_events": (None, [_vp, _vp]),
    "knap_seq_cost": (_d, [_i64, _d, _d]),
    "knap_flux_workload": (_d, [_i64, _i64, _d]),
    "knap_fit_cost_model": (_i, [_pd, _pd, _pd, _i, _pd, _pd, _pd]),
    "knap_parse_topology": (_i, [C.c_char_p, _pi, _i, _pi]),
    "knap_greedy_assign": (_i, [_pi64, _i, _pi, _i, _d, _d, _pi, _pd]),
    "knap_greedy_assign_weights": (_i, [_pd, _i, _pi, _i, _pi, _pd]),
    "knap_chunk_lengths": (_i, [_i64, _i, _pi64]),
    "knap_wir": (_d, [_pd, _pi, _i]),
    "knap_bag_cu_seqlens": (_i, [_pi64, _pi, _i, _i, _pi64, _i, _pi, _pi32]),
}
EXPORTS = tuple(_SIGNATURES)

for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(lib, _name)      # AttributeError here = the library does not export the symbol
    _fn.restype = _res
    _fn.argtypes = _args


class KnapError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        hip = int(lib.knap_last_hip_error()) if code == KNAP_ERR_LAUNCH_FAILED else 0
        extra = f", hipError_t {hip}" if hip else ""
        super().__init__(f"{where}: {knap_strerror(code)} (code {code}{extra})")


def knap_strerror(code: int) -> str:
    return lib.knap_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != KNAP_OK:
        raise KnapError(code, where)


def _ptr(t) -> int:
    """Device (or host) address of a tensor; None -> NULL."""
    return 0 if t is None else int(t.data_ptr())


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


# --------------------------------------------------------------------------- attention

def knap_varlen_attn_fwd(q, k, v, cu_seqlens, n_seq: int, H: int, d: int, scale: float, out, lse,
                         stream=None, check: bool = True) -> int:
    """Enqueue the forward kernel.  q, k, v, out: bf16 (T, H, d) CUDA tensors; cu_seqlens: int32
    (n_seq + 1,) CUDA tensor; lse: fp32 (H, T).  Returns the library's status code."""
    rc = lib.knap_varlen_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), n_seq, H, d, scale,
                                  _ptr(out), _ptr(lse), _stream_handle(stream))
    if check:
        _check(rc, "knap_varlen_attn_fwd")
    return rc


def knap_varlen_attn_bwd_workspace_bytes(total_tokens: int, n_seq: int, H: int, d: int) -> int:
    return int(lib.knap_varlen_attn_bwd_workspace_bytes(total_tokens, n_seq, H, d))


def knap_varlen_attn_bwd(q, k, v, cu_seqlens, n_seq: int, H: int, d: int, scale: float, out, lse, dout,
                         dq, dk, dv, total_tokens: int, workspace, workspace_bytes: Optional[int] = None,
                         stream=None, check: bool = True) -> int:
    """Enqueue the backward kernels.  `workspace` is a CUDA uint8 tensor of at least
    knap_varlen_attn_bwd_workspace_bytes(...) bytes."""
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib.knap_varlen_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), n_seq, H, d, scale,
                                  _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                                  total_tokens, _ptr(workspace), workspace_bytes, _stream_handle(stream))
    if check:
        _check(rc, "knap_varlen_attn_bwd")
    return rc


def knap_varlen_attn_bwd_noalloc(q, k, v, cu_seqlens, n_seq: int, H: int, d: int, scale: float, out, lse, dout,
                                 dq, dk, dv, total_tokens: int, stream=None, check: bool = True) -> int:
    """knap_varlen_attn_bwd without a workspace argument: the scratch is an array in the library's device
    image (total_tokens * H <= KNAP_NOALLOC_MAX_ROWS)."""
    rc = lib.knap_varlen_attn_bwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), n_seq, H, d, scale,
                                          _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                                          total_tokens, _stream_handle(stream))
    if check:
        _check(rc, "knap_varlen_attn_bwd_noalloc")
    return rc


def knap_varlen_attn_causal_fwd(q, k, v, cu_seqlens, n_seq: int, H: int, d: int, scale: float, out, lse,
                                stream=None, check: bool = True) -> int:
    """knap_varlen_attn_fwd with the causal mask inside every sequence."""
    rc = lib.knap_varlen_attn_causal_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), n_seq, H, d, scale,
                                         _ptr(out), _ptr(lse), _stream_handle(stream))
    if check:
        _check(rc, "knap_varlen_attn_causal_fwd")
    return rc


def knap_varlen_attn_causal_bwd(q, k, v, cu_seqlens, n_seq: int, H: int, d: int, scale: float, out, lse, dout,
                                dq, dk, dv, total_tokens: int, workspace, workspace_bytes: Optional[int] = None,
                                stream=None, check: bool = True) -> int:
    """knap_varlen_attn_bwd with the causal mask inside every sequence."""
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib.knap_varlen_attn_causal_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), n_seq, H, d, scale,
                                         _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                                         total_tokens, _ptr(workspace), workspace_bytes, _stream_handle(stream))
    if check:
        _check(rc, "knap_varlen_attn_causal_bwd")
    return rc


def knap_last_hip_error() -> int:
    return int(lib.knap_last_hip_error())


def knap_bwd_profile_events(start: Optional[int], stop: Optional[int]) -> None:
    """Raw hipEvent_t handles (ints) recorded around the main backward kernel; None switches it off."""
    lib.knap_bwd_profile_events(start or 0, stop or 0)


def knap_launch_workgroups(which: int) -> int:
    return int(lib.knap_launch_workgroups(which))


# --------------------------------------------------------------------------- Ulysses layout switch (local part)

def knap_ulysses_pack_heads(x, local_tokens: int, H: int, d: int, g: int, y, stream=None, check: bool = True) -> int:
    """x (T_r, H, d) -> y (g, T_r, H/g, d); CUDA tensors of a two-byte type."""
    rc = lib.knap_ulysses_pack_heads(_ptr(x), local_tokens, H, d, g, _ptr(y), _stream_handle(stream))
    if check:
        _check(rc, "knap_ulysses_pack_heads")
    return rc


def knap_ulysses_unpack_heads(y, local_tokens: int, H: int, d: int, g: int, x, stream=None, check: bool = True) -> int:
    rc = lib.knap_ulysses_unpack_heads(_ptr(y), local_tokens, H, d, g, _ptr(x), _stream_handle(stream))
    if check:
        _check(rc, "knap_ulysses_unpack_heads")
    return rc


def knap_ulysses_plan_workspace_bytes(n_seq: int, g: int) -> int:
    return int(lib.knap_ulysses_plan_workspace_bytes(n_seq, g))


def knap_ulysses_plan(cu_seqlens, n_seq: int, total_tokens: int, g: int, row_map, workspace,
                      workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    """Fills row_map (int32 CUDA tensor of total_tokens entries) for a g-GPU bag."""
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib.knap_ulysses_plan(_ptr(cu_seqlens), n_seq, total_tokens, g, _ptr(row_map), _ptr(workspace),
                               workspace_bytes, _stream_handle(stream))
    if check:
        _check(rc, "knap_ulysses_plan")
    return rc


def knap_ulysses_gather_chunks(recv, row_map, total_tokens: int, heads_local: int, d: int, z,
                               stream=None, check: bool = True) -> int:
    rc = lib.knap_ulysses_gather_chunks(_ptr(recv), _ptr(row_map), total_tokens, heads_local, d, _ptr(z),
                                        _stream_handle(stream))
    if check:
        _check(rc, "knap_ulysses_gather_chunks")
    return rc


def knap_ulysses_scatter_chunks(z, row_map, total_tokens: int, heads_local: int, d: int, send,
                                stream=None, check: bool = True) -> int:
    rc = lib.knap_ulysses_scatter_chunks(_ptr(z), _ptr(row_map), total_tokens, heads_local, d, _ptr(send),
                                         _stream_handle(stream))
    if check:
        _check(rc, "knap_ulysses_scatter_chunks")
    return rc


def knap_ulysses_local_tokens(seq_lens, g: int):
    """T_r for r = 0..g-1: tokens every GPU of a g-GPU bag holds after the second pass."""
    n = len(seq_lens)
    arr = (C.c_int64 * max(n, 1))(*[int(x) for x in seq_lens])
    out = (C.c_int64 * g)()
    _check(lib.knap_ulysses_local_tokens(arr, n, g, out), "knap_ulysses_local_tokens")
    return [int(v) for v in out]


# --------------------------------------------------------------------------- host model / balancer

def knap_seq_cost(L: int, a: float, b: float) -> float:
    return float(lib.knap_seq_cost(L, a, b))


def knap_flux_workload(l: int, d_model: int, gamma: float) -> float:
    return float(lib.knap_flux_workload(l, d_model, gamma))


def _darr(xs: Sequence[float]):
    return (C.c_double * len(xs))(*[float(x) for x in xs])


def _iarr(xs: Sequence[int]):
    return (C.c_int * len(xs))(*[int(x) for x in xs])


def _i64arr(xs: Sequence[int]):
    return (C.c_int64 * len(xs))(*[int(x) for x in xs])


def knap_fit_cost_model(sum_l2: Sequence[float], sum_l: Sequence[float], t: Sequence[float]) -> Tuple[float, float, float]:
    a, b, r = C.c_double(), C.c_double(), C.c_double()
    _check(lib.knap_fit_cost_model(_darr(sum_l2), _darr(sum_l), _darr(t), len(t), C.byref(a), C.byref(b), C.byref(r)),
           "knap_fit_cost_model")
    return a.value, b.value, r.value


def knap_parse_topology(spec: str, cap: int = 4096) -> List[int]:
    bags = (C.c_int * cap)()
    n = C.c_int()
    _check(lib.knap_parse_topology(spec.encode(), bags, cap, C.byref(n)), "knap_parse_topology")
    return list(bags[: n.value])


def knap_greedy_assign(seq_len: Sequence[int], bag_gpus: Sequence[int], a: float, b: float) -> Tuple[List[int], List[float]]:
    bag_of = (C.c_int * max(1, len(seq_len)))()
    load = (C.c_double * len(bag_gpus))()
    _check(lib.knap_greedy_assign(_i64arr(seq_len), len(seq_len), _iarr(bag_gpus), len(bag_gpus), a, b, bag_of, load),
           "knap_greedy_assign")
    return list(bag_of[: len(seq_len)]), list(load)


def knap_greedy_assign_weights(weight: Sequence[float], bag_gpus: Sequence[int]) -> Tuple[List[int], List[float]]:
    bag_of = (C.c_int * max(1, len(weight)))()
    load = (C.c_double * len(bag_gpus))()
    _check(lib.knap_greedy_assign_weights(_darr(weight), len(weight), _iarr(bag_gpus), len(bag_gpus), bag_of, load),
           "knap_greedy_assign_weights")
    return list(bag_of[: len(weight)]), list(load)


def knap_chunk_lengths(L: int, g: int) -> List[int]:
    out = (C.c_int64 * max(1, g))()
    _check(lib.knap_chunk_lengths(L, g, out), "knap_chunk_lengths")
    return list(out[:g])


def knap_wir(bag_load: Sequence[float], bag_gpus: Sequence[int]) -> float:
    return float(lib.knap_wir(_darr(bag_load), _iarr(bag_gpus), len(bag_gpus)))


def knap_bag_cu_seqlens(seq_len: Sequence[int], bag_of_seq: Sequence[int], bag: int) -> Tuple[List[int], List[int]]:
    n = len(seq_len)
    out_len = (C.c_int64 * max(1, n))()
    cu = (C.c_int32 * (n + 1))()
    cnt = C.c_int()
    _check(lib.knap_bag_cu_seqlens(_i64arr(seq_len), _iarr(bag_of_seq), n, bag, out_len, n, C.byref(cnt), cu),
           "knap_bag_cu_seqlens")
    return list(out_len[: cnt.value]), list(cu[: cnt.value + 1])
