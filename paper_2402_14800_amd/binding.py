"""ctypes binding of libmoeprune.so: argument marshalling only.

Every function here has the name and meaning of the C entry point it calls (see
include/moeprune.h); torch supplies device memory and the stream, nothing else.
Importing this module raises if the library has not been built -- there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoeprune.so")

MOEP_F32, MOEP_BF16 = 0, 1
_STATUS = {0: "MOEP_OK", 1: "MOEP_EINVAL", 2: "MOEP_EUNSUPPORTED", 3: "MOEP_EWORKSPACE", 4: "MOEP_EHIP"}

EXPORTS = (
    "moep_num_subsets", "moep_subset_unrank", "moep_subset_rank", "moep_last_error",
    "moe_expert_outputs_workspace", "moe_expert_outputs",
    "prune_enumerate_workspace", "prune_enumerate",
    "prune_enumerate_multi_workspace", "prune_enumerate_multi", "prune_enumerate_static",
    "prune_enumerate_direct_workspace", "prune_enumerate_direct",
    "moe_forward_skip_workspace", "moe_forward_skip", "moe_forward_pruned_skip",
    "moe_packed_weights_bytes", "moe_pack_weights", "moe_forward_pruned_skip_packed",
    "moe_expert_outputs_packed_workspace", "moe_expert_outputs_packed",
    "moe_forward_skip_topk_workspace", "moe_forward_skip_topk",
    "skip_calibrate_beta_workspace", "skip_calibrate_beta", "expert_selection_stats",
    "moe_expert_outputs_ranked_workspace", "moe_expert_outputs_ranked", "prune_enumerate_ranked",
    "moep_timing_enable", "moep_timing_collect", "moep_timing_records", "moep_mfma_ceiling",
)


class MoepError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2402_14800_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.moep_num_subsets.restype = c_int64
    lib.moep_num_subsets.argtypes = [c_int, c_int]
    lib.moep_subset_unrank.restype = c_int
    lib.moep_subset_unrank.argtypes = [c_int, c_int, c_int64, POINTER(c_uint32)]
    lib.moep_subset_rank.restype = c_int64
    lib.moep_subset_rank.argtypes = [c_int, c_int, c_uint32]
    lib.moep_last_error.restype = c_char_p
    lib.moep_last_error.argtypes = []
    lib.moe_expert_outputs_workspace.restype = c_size_t
    lib.moe_expert_outputs_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int]
    lib.moe_expert_outputs.restype = c_int
    lib.moe_expert_outputs.argtypes = [c_void_p] * 5 + [c_int64, c_int, c_int, c_int, c_int,
                                                        c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.prune_enumerate_workspace.restype = c_size_t
    lib.prune_enumerate_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int, c_int]
    lib.prune_enumerate.restype = c_int
    lib.prune_enumerate.argtypes = [c_void_p, c_void_p, c_int64, c_int, c_int, c_int, c_int, c_int,
                                    c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.prune_enumerate_direct_workspace.restype = c_size_t
    lib.prune_enumerate_direct_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int, c_int]
    lib.prune_enumerate_direct.restype = c_int
    lib.prune_enumerate_direct.argtypes = lib.prune_enumerate.argtypes
    lib.prune_enumerate_static.restype = c_int
    lib.prune_enumerate_static.argtypes = [c_void_p, c_void_p, c_int64, c_int, c_int, c_int, c_int, c_int,
                                           c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.prune_enumerate_multi_workspace.restype = c_size_t
    lib.prune_enumerate_multi_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int, POINTER(c_int), c_int]
    lib.prune_enumerate_multi.restype = c_int
    lib.prune_enumerate_multi.argtypes = [c_void_p, c_void_p, c_int64, c_int, c_int, c_int, c_int, c_int,
                                          POINTER(c_int), c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_size_t, c_void_p]
    lib.moe_forward_skip_workspace.restype = c_size_t
    lib.moe_forward_skip_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int]
    lib.moe_forward_skip.restype = c_int
    lib.moe_forward_skip.argtypes = [c_void_p] * 5 + [c_int64, c_int, c_int, c_int, c_int, c_int, c_float,
                                                      c_void_p, c_void_p, c_void_p, c_void_p,
                                                      c_void_p, c_size_t, c_void_p]
    lib.moe_forward_pruned_skip.restype = c_int
    lib.moe_forward_pruned_skip.argtypes = [c_void_p] * 5 + [c_int64, c_int, c_int, c_int, c_int, c_int, c_uint32,
                                                             c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                                             c_void_p, c_size_t, c_void_p]
    lib.moe_packed_weights_bytes.restype = c_size_t
    lib.moe_packed_weights_bytes.argtypes = [c_int, c_int, c_int, c_int]
    lib.moe_pack_weights.restype = c_int
    lib.moe_pack_weights.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
    lib.moe_expert_outputs_packed_workspace.restype = c_size_t
    lib.moe_expert_outputs_packed_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int]
    lib.moe_expert_outputs_packed.restype = c_int
    lib.moe_expert_outputs_packed.argtypes = [c_void_p] * 3 + [c_int64, c_int, c_int, c_int, c_int,
                                                               c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.moe_forward_pruned_skip_packed.restype = c_int
    lib.moe_forward_pruned_skip_packed.argtypes = [c_void_p] * 3 + [c_int64, c_int, c_int, c_int, c_int, c_int, c_uint32,
                                                                    c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                                                    c_void_p, c_size_t, c_void_p]
    lib.moe_forward_skip_topk_workspace.restype = c_size_t
    lib.moe_forward_skip_topk_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int, c_int]
    lib.moe_forward_skip_topk.restype = c_int
    lib.moe_forward_skip_topk.argtypes = [c_void_p] * 5 + [c_int64, c_int, c_int, c_int, c_int, c_int, c_uint32,
                                                           c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                                           c_void_p, c_size_t, c_void_p]
    lib.skip_calibrate_beta_workspace.restype = c_size_t
    lib.skip_calibrate_beta_workspace.argtypes = [c_int64]
    lib.skip_calibrate_beta.restype = c_int
    lib.skip_calibrate_beta.argtypes = [c_void_p, c_int64, c_int, c_uint32, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.expert_selection_stats.restype = c_int
    lib.expert_selection_stats.argtypes = [c_void_p, c_int64, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                           c_void_p]
    lib.moe_expert_outputs_ranked_workspace.restype = c_size_t
    lib.moe_expert_outputs_ranked_workspace.argtypes = [c_int64, c_int, c_int, c_int, c_int, c_int]
    lib.moe_expert_outputs_ranked.restype = c_int
    lib.moe_expert_outputs_ranked.argtypes = [c_void_p] * 5 + [c_int64, c_int, c_int, c_int, c_int, c_int,
                                                               c_void_p, c_void_p, c_void_p, c_void_p,
                                                               c_void_p, c_size_t, c_void_p]
    lib.prune_enumerate_ranked.restype = c_int
    lib.prune_enumerate_ranked.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int, c_int, c_int,
                                           c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_size_t, c_void_p]
    lib.moep_timing_enable.restype = c_int
    lib.moep_timing_enable.argtypes = [c_int]
    lib.moep_timing_collect.restype = c_int
    lib.moep_timing_collect.argtypes = [POINTER(c_char_p), POINTER(c_double), POINTER(c_int64), c_int]
    lib.moep_timing_records.restype = c_int
    lib.moep_timing_records.argtypes = [POINTER(c_char_p), POINTER(c_float), c_int]
    lib.moep_mfma_ceiling.restype = c_int
    lib.moep_mfma_ceiling.argtypes = [c_void_p, c_void_p, c_size_t, c_int, c_void_p, c_size_t, POINTER(c_double),
                                      c_void_p]
    return lib


_lib = _load()


def _check(status: int) -> None:
    if status != 0:
        raise MoepError(status, _lib.moep_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOEP_F32
    if t.dtype == torch.bfloat16:
        return MOEP_BF16
    raise TypeError(f"unsupported storage dtype {t.dtype}: use float32 or bfloat16")


def _dev(*tensors: torch.Tensor) -> torch.device:
    d = tensors[0].device
    for t in tensors:
        if t.device != d or t.device.type != "cuda":
            raise ValueError("all tensors must live on the same GPU")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous (row-major)")
    return d


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(dev: torch.device):
    return c_void_p(torch.cuda.current_stream(dev).cuda_stream)


def _workspace(nbytes: int, dev: torch.device, ws: Optional[torch.Tensor]) -> torch.Tensor:
    if ws is not None:
        if ws.dtype != torch.uint8 or ws.device != dev or not ws.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 tensor on the same GPU")
        return ws
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)


# ---------------------------------------------------------------- host helpers
def num_subsets(E: int, r: int) -> int:
    return int(_lib.moep_num_subsets(E, r))


def subset_unrank(E: int, r: int, idx: int) -> int:
    m = c_uint32(0)
    _check(_lib.moep_subset_unrank(E, r, idx, ctypes.byref(m)))
    return int(m.value)


def subset_rank(E: int, r: int, mask: int) -> int:
    return int(_lib.moep_subset_rank(E, r, mask))


# ---------------------------------------------------------------- entry points
def moe_expert_outputs_workspace(T: int, E: int, H: int, F: int, dtype_code: int) -> int:
    return int(_lib.moe_expert_outputs_workspace(T, E, H, F, dtype_code))


def moe_expert_outputs(x, Wgate, W1, W3, W2, logits=None, Y=None, workspace=None):
    """logits [T,E] fp32 and Y [E,T,H] for every expert and token (asynchronous on the current stream)."""
    dev = _dev(x, Wgate, W1, W3, W2)
    dt = _dtype_code(x)
    T, H = x.shape
    E, F, _ = W1.shape
    assert Wgate.shape == (E, H) and W3.shape == (E, F, H) and W2.shape == (E, H, F)
    assert all(_dtype_code(t) == dt for t in (Wgate, W1, W3, W2))
    if logits is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    if Y is None:
        Y = torch.empty((E, T, H), dtype=x.dtype, device=dev)
    need = _lib.moe_expert_outputs_workspace(T, E, H, F, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.moe_expert_outputs(_ptr(x), _ptr(Wgate), _ptr(W1), _ptr(W3), _ptr(W2), T, E, H, F, dt,
                                   _ptr(logits), _ptr(Y), _ptr(ws), ws.numel(), _stream(dev)))
    return logits, Y


def prune_enumerate_workspace(T: int, E: int, H: int, k: int, r: int, dtype_code: int) -> int:
    return int(_lib.prune_enumerate_workspace(T, E, H, k, r, dtype_code))


def prune_enumerate(logits, Y, k: int, r: int, workspace=None, count_unaffected: bool = True):
    """loss [C(E,r)] fp32, argmin [1] int32, argmin_mask [1] (int32 view of the uint32 mask),
    unaffected_pairs [1] int64 (or None).  Device tensors; asynchronous on the current stream."""
    dev = _dev(logits, Y)
    dt = _dtype_code(Y)
    E, T, H = Y.shape
    assert logits.shape == (T, E) and logits.dtype == torch.float32
    n = num_subsets(E, r)
    if n < 0:
        raise MoepError(1, f"r={r} out of range [1, E={E}]")
    loss = torch.empty((n,), dtype=torch.float32, device=dev)
    argmin = torch.empty((1,), dtype=torch.int32, device=dev)
    amask = torch.empty((1,), dtype=torch.int32, device=dev)
    unaffected = torch.empty((1,), dtype=torch.int64, device=dev) if count_unaffected else None
    need = _lib.prune_enumerate_workspace(T, E, H, k, r, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.prune_enumerate(_ptr(logits), _ptr(Y), T, E, H, dt, k, r, _ptr(loss), _ptr(argmin),
                                _ptr(amask), _ptr(unaffected), _ptr(ws), ws.numel(), _stream(dev)))
    return loss, argmin, amask, unaffected


def prune_enumerate_direct(logits, Y, k: int, r: int, workspace=None, count_unaffected: bool = True):
    """prune_enumerate's outputs from Eq. 3 as written (no Gram matrices); at most 128 subsets, k <= 4."""
    dev = _dev(logits, Y)
    dt = _dtype_code(Y)
    E, T, H = Y.shape
    assert logits.shape == (T, E) and logits.dtype == torch.float32
    n = num_subsets(E, r)
    if n < 0:
        raise MoepError(1, f"r={r} out of range [1, E={E}]")
    loss = torch.empty((n,), dtype=torch.float32, device=dev)
    argmin = torch.empty((1,), dtype=torch.int32, device=dev)
    amask = torch.empty((1,), dtype=torch.int32, device=dev)
    unaffected = torch.empty((1,), dtype=torch.int64, device=dev) if count_unaffected else None
    need = _lib.prune_enumerate_direct_workspace(T, E, H, k, r, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.prune_enumerate_direct(_ptr(logits), _ptr(Y), T, E, H, dt, k, r, _ptr(loss), _ptr(argmin),
                                       _ptr(amask), _ptr(unaffected), _ptr(ws), ws.numel(), _stream(dev)))
    return loss, argmin, amask, unaffected


STATIC_SCRATCH_BYTES = 32 << 20      # MOEP_STATIC_SCRATCH_BYTES of include/moeprune.h


def prune_enumerate_static(logits, Y, k: int, r: int, out=None, count_unaffected: bool = True):
    """prune_enumerate on the library's built-in scratch array: no workspace, nothing allocated by the call
    when `out` carries the four output tensors (loss, argmin, argmin_mask, unaffected_pairs)."""
    dev = _dev(logits, Y)
    dt = _dtype_code(Y)
    E, T, H = Y.shape
    assert logits.shape == (T, E) and logits.dtype == torch.float32
    if out is None:
        n = num_subsets(E, r)
        if n < 0:
            raise MoepError(1, f"r={r} out of range [1, E={E}]")
        out = (torch.empty((n,), dtype=torch.float32, device=dev), torch.empty((1,), dtype=torch.int32, device=dev),
               torch.empty((1,), dtype=torch.int32, device=dev),
               torch.empty((1,), dtype=torch.int64, device=dev) if count_unaffected else None)
    loss, argmin, amask, unaffected = out
    _check(_lib.prune_enumerate_static(_ptr(logits), _ptr(Y), T, E, H, dt, k, r, _ptr(loss), _ptr(argmin),
                                       _ptr(amask), _ptr(unaffected), _stream(dev)))
    return loss, argmin, amask, unaffected


def prune_enumerate_multi_workspace(T: int, E: int, H: int, k: int, rs, dtype_code: int) -> int:
    arr = (c_int * len(rs))(*rs)
    return int(_lib.prune_enumerate_multi_workspace(T, E, H, k, len(rs), arr, dtype_code))


def prune_enumerate_multi(logits, Y, k: int, rs, workspace=None, count_unaffected: bool = True):
    """prune_enumerate for every r of `rs` with one pass over Y.  Returns a list of
    (loss [C(E,r)], argmin [1], argmin_mask [1], unaffected_pairs [1] or None), one per r (views)."""
    dev = _dev(logits, Y)
    dt = _dtype_code(Y)
    E, T, H = Y.shape
    assert logits.shape == (T, E) and logits.dtype == torch.float32
    rs = [int(r) for r in rs]
    ns = [num_subsets(E, r) for r in rs]
    if not rs or min(ns) < 0:
        raise MoepError(1, f"rs={rs}: every r must lie in [1, E={E}]")
    loss = torch.empty((sum(ns),), dtype=torch.float32, device=dev)
    argmin = torch.empty((len(rs),), dtype=torch.int32, device=dev)
    amask = torch.empty((len(rs),), dtype=torch.int32, device=dev)
    unaffected = torch.empty((len(rs),), dtype=torch.int64, device=dev) if count_unaffected else None
    arr = (c_int * len(rs))(*rs)
    need = _lib.prune_enumerate_multi_workspace(T, E, H, k, len(rs), arr, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.prune_enumerate_multi(_ptr(logits), _ptr(Y), T, E, H, dt, k, len(rs), arr, _ptr(loss), _ptr(argmin),
                                      _ptr(amask), _ptr(unaffected), _ptr(ws), ws.numel(), _stream(dev)))
    out, off = [], 0
    for i, n in enumerate(ns):
        out.append((loss[off:off + n], argmin[i:i + 1], amask[i:i + 1],
                    unaffected[i:i + 1] if unaffected is not None else None))
        off += n
    return out


def moe_expert_outputs_ranked(x, Wgate, W1, W3, W2, n_rank: int, workspace=None, out=None):
    """logits [T,E] fp32, ranked_experts [T,n_rank] int32, slot_of [T,n_rank] int32, Yr [T*n_rank,H].
    `out` may carry a previous call's (logits, ranked_experts, slot_of, Yr) to be overwritten."""
    dev = _dev(x, Wgate, W1, W3, W2)
    dt = _dtype_code(x)
    T, H = x.shape
    E, F, _ = W1.shape
    assert Wgate.shape == (E, H) and W3.shape == (E, F, H) and W2.shape == (E, H, F)
    if out is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=dev)
        experts = torch.empty((T, max(n_rank, 1)), dtype=torch.int32, device=dev)
        slot_of = torch.empty((T, max(n_rank, 1)), dtype=torch.int32, device=dev)
        Yr = torch.empty((T * max(n_rank, 1), H), dtype=x.dtype, device=dev)
    else:
        logits, experts, slot_of, Yr = out
    need = _lib.moe_expert_outputs_ranked_workspace(T, E, H, F, dt, n_rank)
    ws = _workspace(need, dev, workspace)
    _check(_lib.moe_expert_outputs_ranked(_ptr(x), _ptr(Wgate), _ptr(W1), _ptr(W3), _ptr(W2), T, E, H, F, dt,
                                          n_rank, _ptr(logits), _ptr(experts), _ptr(slot_of), _ptr(Yr),
                                          _ptr(ws), ws.numel(), _stream(dev)))
    return logits, experts, slot_of, Yr


def prune_enumerate_ranked(logits, experts, slot_of, Yr, k: int, r: int, workspace=None,
                           count_unaffected: bool = True):
    """As prune_enumerate, from the outputs of moe_expert_outputs_ranked."""
    dev = _dev(logits, Yr)
    dt = _dtype_code(Yr)
    T, E = logits.shape
    n_rank = experts.shape[1]
    H = Yr.shape[1]
    n_sub = num_subsets(E, r)
    if n_sub < 0:
        raise MoepError(1, f"r={r} out of range for E={E}")
    loss = torch.empty((n_sub,), dtype=torch.float32, device=dev)
    argmin = torch.empty((1,), dtype=torch.int32, device=dev)
    amask = torch.empty((1,), dtype=torch.int32, device=dev)
    unaff = torch.empty((1,), dtype=torch.int64, device=dev) if count_unaffected else None
    need = _lib.prune_enumerate_workspace(T, E, H, k, r, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.prune_enumerate_ranked(_ptr(logits), _ptr(experts), _ptr(slot_of), _ptr(Yr), T, E, H, dt, n_rank,
                                       k, r, _ptr(loss), _ptr(argmin), _ptr(amask), _ptr(unaff), _ptr(ws),
                                       ws.numel(), _stream(dev)))
    return loss, argmin, amask, unaff


def moe_forward_skip_workspace(T: int, E: int, H: int, F: int, dtype_code: int) -> int:
    return int(_lib.moe_forward_skip_workspace(T, E, H, F, dtype_code))


def moe_forward_skip(x, Wgate, W1, W3, W2, beta: float, k: int = 2, workspace=None,
                     want_logits: bool = True, want_top2: bool = True, kept_mask: Optional[int] = None):
    """out [T,H], skip_mask [T] uint8, logits [T,E] fp32 (or None), top2 [T,2] int32 (or None).
    With `kept_mask` the call goes to moe_forward_pruned_skip (top-2 among the kept experts)."""
    dev = _dev(x, Wgate, W1, W3, W2)
    dt = _dtype_code(x)
    T, H = x.shape
    E, F, _ = W1.shape
    assert Wgate.shape == (E, H) and W3.shape == (E, F, H) and W2.shape == (E, H, F)
    out = torch.empty((T, H), dtype=x.dtype, device=dev)
    skip = torch.empty((T,), dtype=torch.uint8, device=dev)
    logits = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    top2 = torch.empty((T, 2), dtype=torch.int32, device=dev) if want_top2 else None
    need = _lib.moe_forward_skip_workspace(T, E, H, F, dt)
    ws = _workspace(need, dev, workspace)
    if kept_mask is None:
        _check(_lib.moe_forward_skip(_ptr(x), _ptr(Wgate), _ptr(W1), _ptr(W3), _ptr(W2), T, E, H, F, dt, k,
                                     c_float(beta), _ptr(out), _ptr(skip), _ptr(logits), _ptr(top2),
                                     _ptr(ws), ws.numel(), _stream(dev)))
    else:
        _check(_lib.moe_forward_pruned_skip(_ptr(x), _ptr(Wgate), _ptr(W1), _ptr(W3), _ptr(W2), T, E, H, F, dt, k,
                                            c_uint32(kept_mask), c_float(beta), _ptr(out), _ptr(skip),
                                            _ptr(logits), _ptr(top2), _ptr(ws), ws.numel(), _stream(dev)))
    return out, skip, logits, top2


def moe_forward_pruned_skip(x, Wgate, W1, W3, W2, kept_mask: int, beta: float, **kw):
    return moe_forward_skip(x, Wgate, W1, W3, W2, beta, kept_mask=kept_mask, **kw)


def moe_pack_weights(W1, W3, W2) -> torch.Tensor:
    """The layer's expert weights in the layout the bf16 GEMMs read (uint8 tensor, for *_packed calls)."""
    dev = _dev(W1, W3, W2)
    dt = _dtype_code(W1)
    E, F, H = W1.shape
    assert W3.shape == (E, F, H) and W2.shape == (E, H, F)
    need = int(_lib.moe_packed_weights_bytes(E, H, F, dt))
    if need == 0:
        raise MoepError(2, "moe_pack_weights: bf16 weights with H and F multiples of 64 only")
    packed = torch.empty((need,), dtype=torch.uint8, device=dev)
    _check(_lib.moe_pack_weights(_ptr(W1), _ptr(W3), _ptr(W2), E, H, F, dt, _ptr(packed), _stream(dev)))
    return packed


def moe_expert_outputs_packed(x, Wgate, packed, F: int, logits=None, Y=None, workspace=None):
    """moe_expert_outputs on weights packed once by moe_pack_weights."""
    dev = _dev(x, Wgate, packed)
    dt = _dtype_code(x)
    T, H = x.shape
    E = Wgate.shape[0]
    assert Wgate.shape == (E, H) and packed.numel() == int(_lib.moe_packed_weights_bytes(E, H, F, dt))
    if logits is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    if Y is None:
        Y = torch.empty((E, T, H), dtype=x.dtype, device=dev)
    need = _lib.moe_expert_outputs_packed_workspace(T, E, H, F, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.moe_expert_outputs_packed(_ptr(x), _ptr(Wgate), _ptr(packed), T, E, H, F, dt, _ptr(logits), _ptr(Y),
                                          _ptr(ws), ws.numel(), _stream(dev)))
    return logits, Y


def moe_forward_pruned_skip_packed(x, Wgate, packed, F: int, beta: float, kept_mask: Optional[int] = None,
                                   k: int = 2, workspace=None, want_logits: bool = True, want_top2: bool = True):
    """moe_forward_pruned_skip on weights packed once by moe_pack_weights."""
    dev = _dev(x, Wgate, packed)
    dt = _dtype_code(x)
    T, H = x.shape
    E = Wgate.shape[0]
    assert Wgate.shape == (E, H) and packed.numel() == int(_lib.moe_packed_weights_bytes(E, H, F, dt))
    if kept_mask is None:
        kept_mask = (1 << E) - 1
    out = torch.empty((T, H), dtype=x.dtype, device=dev)
    skip = torch.empty((T,), dtype=torch.uint8, device=dev)
    logits = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    top2 = torch.empty((T, 2), dtype=torch.int32, device=dev) if want_top2 else None
    need = _lib.moe_forward_skip_workspace(T, E, H, F, dt)
    ws = _workspace(need, dev, workspace)
    _check(_lib.moe_forward_pruned_skip_packed(_ptr(x), _ptr(Wgate), _ptr(packed), T, E, H, F, dt, k,
                                               c_uint32(kept_mask), c_float(beta), _ptr(out), _ptr(skip),
                                               _ptr(logits), _ptr(top2), _ptr(ws), ws.numel(), _stream(dev)))
    return out, skip, logits, top2


def moe_forward_skip_topk(x, Wgate, W1, W3, W2, k: int, beta: float, kept_mask: Optional[int] = None,
                          workspace=None, want_logits: bool = True, want_topk: bool = True):
    """out [T,H], n_used [T] int32 (i* per token), logits [T,E] fp32 (or None), topk [T,k] int32 (or None)."""
    dev = _dev(x, Wgate, W1, W3, W2)
    dt = _dtype_code(x)
    T, H = x.shape
    E, F, _ = W1.shape
    assert Wgate.shape == (E, H) and W3.shape == (E, F, H) and W2.shape == (E, H, F)
    if kept_mask is None:
        kept_mask = (1 << E) - 1
    out = torch.empty((T, H), dtype=x.dtype, device=dev)
    n_used = torch.empty((T,), dtype=torch.int32, device=dev)
    logits = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    topk = torch.empty((T, max(k, 1)), dtype=torch.int32, device=dev) if want_topk else None
    need = _lib.moe_forward_skip_topk_workspace(T, E, H, F, dt, k)
    ws = _workspace(need, dev, workspace)
    _check(_lib.moe_forward_skip_topk(_ptr(x), _ptr(Wgate), _ptr(W1), _ptr(W3), _ptr(W2), T, E, H, F, dt, k,
                                      c_uint32(kept_mask), c_float(beta), _ptr(out), _ptr(n_used),
                                      _ptr(logits), _ptr(topk), _ptr(ws), ws.numel(), _stream(dev)))
    return out, n_used, logits, topk


def skip_calibrate_beta(logits, kept_mask: Optional[int] = None, workspace=None) -> torch.Tensor:
    """beta [1] fp32 on the device: the median of w_e1 / w_e0 over the rows of logits [T,E]."""
    dev = _dev(logits)
    assert logits.dtype == torch.float32 and logits.dim() == 2
    T, E = logits.shape
    if kept_mask is None:
        kept_mask = (1 << E) - 1
    beta = torch.empty((1,), dtype=torch.float32, device=dev)
    need = _lib.skip_calibrate_beta_workspace(T)
    ws = _workspace(need, dev, workspace)
    _check(_lib.skip_calibrate_beta(_ptr(logits), T, E, c_uint32(kept_mask), _ptr(beta), _ptr(ws), ws.numel(),
                                    _stream(dev)))
    return beta


def expert_selection_stats(logits, k: int, r: Optional[int] = None):
    """count [E] int64, coselect [E,E] int64, frequency_mask (int32 view of the uint32 mask, [1]) or None."""
    dev = _dev(logits)
    assert logits.dtype == torch.float32 and logits.dim() == 2
    T, E = logits.shape
    count = torch.empty((E,), dtype=torch.int64, device=dev)
    co = torch.empty((E, E), dtype=torch.int64, device=dev)
    fmask = torch.empty((1,), dtype=torch.int32, device=dev) if r is not None else None
    _check(_lib.expert_selection_stats(_ptr(logits), T, E, k, r if r is not None else 0, _ptr(count), _ptr(co),
                                       _ptr(fmask), _stream(dev)))
    return count, co, fmask


# ---------------------------------------------------------------- kernel timing
def kernel_timing_enable(on: bool = True) -> None:
    _check(_lib.moep_timing_enable(1 if on else 0))


def kernel_timing_collect() -> Dict[str, Tuple[float, int]]:
    """{kernel name: (total milliseconds, launches)} since the last collect; waits for the GPU."""
    cap = 64
    names = (c_char_p * cap)()
    ms = (c_double * cap)()
    cnt = (c_int64 * cap)()
    n = _lib.moep_timing_collect(names, ms, cnt, cap)
    if n < 0:
        raise MoepError(4, _lib.moep_last_error().decode())
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


def kernel_timing_records():
    """[(kernel name, milliseconds)] launch by launch since the last collect; waits for the GPU."""
    cap = 8192
    names = (c_char_p * cap)()
    ms = (c_float * cap)()
    n = _lib.moep_timing_records(names, ms, cap)
    if n < 0:
        raise MoepError(4, _lib.moep_last_error().decode())
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def mfma_ceiling(a_src: torch.Tensor, b_src: torch.Tensor, steps: int, sink: Optional[torch.Tensor] = None) -> float:
    """Enqueues the MFMA-only launch (operand bits from the two bf16 tensors) and returns its flop count."""
    dev = _dev(a_src, b_src)
    if sink is None:
        sink = torch.empty((1 << 17,), dtype=torch.float32, device=dev)
    flop = c_double(0.0)
    nbytes = min(a_src.numel() * a_src.element_size(), b_src.numel() * b_src.element_size())
    _check(_lib.moep_mfma_ceiling(_ptr(a_src), _ptr(b_src), nbytes, steps, _ptr(sink), sink.numel(),
                                  ctypes.byref(flop), _stream(dev)))
    return float(flop.value)


def kernel_timing_reset() -> None:
    kernel_timing_collect()
