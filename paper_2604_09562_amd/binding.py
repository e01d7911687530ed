"""Thin ctypes binding of libspecverify.so: argument marshalling only.

Every step of the path runs inside the HIP library; PyTorch is used here for
device memory and the current stream.  There is no fallback: if the library is
not built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecverify.so")

SS_F32, SS_BF16, SS_FP8_E4M3 = 0, 1, 2
SS_MAX_DEPTH = 20
SS_OUT_WIDTH = SS_MAX_DEPTH + 1
_DT = {"f32": SS_F32, "bf16": SS_BF16, "fp8": SS_FP8_E4M3}

EXPORTS = ("ss_version", "ss_last_error", "ss_spec_verify_attn_workspace", "ss_spec_verify_attn",
           "ss_spec_accept_workspace", "ss_spec_accept", "ss_spec_accept_static", "ss_spec_accept_static_capacity",
           "ss_spec_accept_tree_greedy", "ss_spec_accept_tree_sample_workspace",
           "ss_spec_accept_tree_sample", "ss_kv_append", "ss_kv_compact", "ss_kv_commit", "ss_depth_init",
           "ss_depth_update", "ss_route_select", "ss_set_option",
           "ss_profile_begin", "ss_profile_collect")


class SpecVerifyError(RuntimeError):
    pass


class ss_paged_kv(ctypes.Structure):
    _fields_ = [("num_blocks", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p)]


class ss_batch(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
                ("max_q_len", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("kv_len", ctypes.c_void_p), ("q_indptr", ctypes.c_void_p),
                ("tree_mask", ctypes.c_void_p)]


SS_FLOW_MAX = 64


class ss_depth_state(ctypes.Structure):
    _fields_ = [("h", ctypes.c_int32), ("idx", ctypes.c_int32), ("f", ctypes.c_double * SS_FLOW_MAX),
                ("d_base", ctypes.c_double), ("gamma", ctypes.c_double), ("d_min", ctypes.c_double),
                ("d_max", ctypes.c_double), ("tau_target", ctypes.c_double), ("tau_recent", ctypes.c_double)]


class ss_worker_metrics(ctypes.Structure):
    _fields_ = [("cache_hit", ctypes.c_double), ("mem", ctypes.c_double), ("load", ctypes.c_double),
                ("queue_depth", ctypes.c_int32), ("stale", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (build it first with ``python -m paper_2604_09562_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SpecVerifyError(f"{LIB_PATH} is not built; run `python -m paper_2604_09562_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.ss_version.restype = ctypes.c_int32
        L.ss_last_error.restype = ctypes.c_char_p
        L.ss_spec_verify_attn_workspace.restype = ctypes.c_size_t
        L.ss_spec_verify_attn_workspace.argtypes = [ctypes.POINTER(ss_paged_kv), ctypes.POINTER(ss_batch),
                                                    ctypes.c_int32, ctypes.c_int32]
        L.ss_spec_verify_attn.restype = ctypes.c_int32
        L.ss_spec_verify_attn.argtypes = [ctypes.POINTER(ss_paged_kv), ctypes.POINTER(ss_batch), ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                          ctypes.c_void_p]
        L.ss_spec_accept_workspace.restype = ctypes.c_size_t
        L.ss_spec_accept_workspace.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.ss_spec_accept.restype = ctypes.c_int32
        L.ss_spec_accept.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                     ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.ss_spec_accept_static.restype = ctypes.c_int32
        L.ss_spec_accept_static.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_float, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_void_p]
        L.ss_spec_accept_static_capacity.restype = ctypes.c_size_t
        L.ss_spec_accept_static_capacity.argtypes = []
        L.ss_kv_append.restype = ctypes.c_int32
        L.ss_spec_accept_tree_greedy.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                                 ctypes.c_int32, ctypes.c_int32] + [ctypes.c_void_p] * 8 + [ctypes.c_size_t,
                                                                                           ctypes.c_void_p]
        L.ss_spec_accept_tree_greedy.restype = ctypes.c_int32
        L.ss_kv_append.argtypes = [ctypes.POINTER(ss_paged_kv), ctypes.POINTER(ss_batch), ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        L.ss_kv_commit.restype = ctypes.c_int32
        L.ss_spec_accept_tree_sample_workspace.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.ss_spec_accept_tree_sample_workspace.restype = ctypes.c_size_t
        L.ss_spec_accept_tree_sample.argtypes = ([ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_int32] + [ctypes.c_void_p] * 8 + [ctypes.c_float] +
                                                 [ctypes.c_void_p] * 5 + [ctypes.c_size_t, ctypes.c_void_p])
        L.ss_spec_accept_tree_sample.restype = ctypes.c_int32
        L.ss_kv_compact.argtypes = [ctypes.POINTER(ss_paged_kv), ctypes.POINTER(ss_batch), ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        L.ss_kv_compact.restype = ctypes.c_int32
        L.ss_kv_commit.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.ss_depth_init.restype = ctypes.c_int32
        L.ss_depth_init.argtypes = [ctypes.POINTER(ss_depth_state)]
        L.ss_depth_update.restype = ctypes.c_int32
        L.ss_depth_update.argtypes = [ctypes.POINTER(ss_depth_state), ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32),
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
        L.ss_route_select.restype = ctypes.c_int32
        L.ss_route_select.argtypes = [ctypes.POINTER(ss_worker_metrics), ctypes.c_int32, ctypes.POINTER(ctypes.c_double),
                                      ctypes.c_double, ctypes.c_double, ctypes.POINTER(ctypes.c_int32)]
        L.ss_set_option.restype = ctypes.c_int32
        L.ss_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int64]
        L.ss_profile_begin.restype = ctypes.c_int32
        L.ss_profile_begin.argtypes = [ctypes.c_int32]
        L.ss_profile_collect.restype = ctypes.c_int32
        L.ss_profile_collect.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise SpecVerifyError(f"specverify error {rc}: {lib().ss_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def ss_version() -> int:
    return int(lib().ss_version())


def ss_set_option(name: str, value: int) -> None:
    _check(lib().ss_set_option(name.encode(), int(value)))


def ss_profile_begin(max_calls: int) -> None:
    _check(lib().ss_profile_begin(int(max_calls)))


def ss_profile_collect(cap: int) -> np.ndarray:
    buf = (ctypes.c_float * max(cap, 1))()
    n = lib().ss_profile_collect(buf, int(cap))
    return np.array(buf[:n], dtype=np.float64)


# --------------------------------------------------------------------------------------------
# device-resident batches
# --------------------------------------------------------------------------------------------
def _to_dev(a: Optional[np.ndarray], device) -> Optional[torch.Tensor]:
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:  # bf16 bits
        return torch.from_numpy(a.view(np.int16)).to(device)
    if a.dtype == np.uint32:  # bit masks
        return torch.from_numpy(a.view(np.int32)).to(device)
    return torch.from_numpy(a).to(device)


to_device = _to_dev   # one array (numpy storage format) -> device tensor, bytes unchanged


def attention_to_device(inp: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    """Copy one attention batch (dict of numpy storage arrays) to the GPU, bytes unchanged."""
    d = dict(inp)
    for name in ("k_cache", "v_cache", "k_scale", "v_scale", "block_table", "kv_len", "q_indptr", "q"):
        d[name] = _to_dev(inp[name], device)
    if inp.get("tree_mask") is not None:
        d["tree_mask"] = _to_dev(inp["tree_mask"], device)
    return d


def append_to_device(inp: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    """Copy one kv_append batch (attention batch + new keys/values) to the GPU, bytes unchanged."""
    d = attention_to_device(inp, device)
    for name in ("k_new", "v_new"):
        d[name] = _to_dev(inp[name], device)
    return d


def accept_to_device(inp: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    d = dict(inp)
    for name in ("q_indptr", "target_logits", "draft_logits", "draft_tokens", "u_accept", "u_sample", "temperature"):
        d[name] = _to_dev(inp[name], device)
    if inp.get("tree_parent") is not None:
        d["tree_parent"] = _to_dev(inp["tree_parent"], device)
    return d


SS_BATCH_REUSE_PLAN = 1


def _descriptors(d: Dict[str, object], max_q_len: int, flags: int = 0):
    kv = ss_paged_kv(d["num_blocks"], d["block_size"], d["num_kv_heads"], d["head_dim"], _DT[d["kv_dtype"]],
                     d["k_cache"].data_ptr(), d["v_cache"].data_ptr(),
                     0 if d["k_scale"] is None else d["k_scale"].data_ptr(),
                     0 if d["v_scale"] is None else d["v_scale"].data_ptr())
    bt = ss_batch(d["batch"], d["max_blocks_per_seq"], max_q_len, flags, d["block_table"].data_ptr(),
                  d["kv_len"].data_ptr(), d["q_indptr"].data_ptr(),
                  d["tree_mask"].data_ptr() if d.get("tree_mask") is not None else 0)
    return kv, bt


def ss_spec_verify_attn_workspace(d: Dict[str, object], max_q_len: int = 0) -> int:
    kv, bt = _descriptors(d, max_q_len)
    n = lib().ss_spec_verify_attn_workspace(ctypes.byref(kv), ctypes.byref(bt), d["num_q_heads"], d["total_rows"])
    if n == 0 and d["batch"] > 0:
        raise SpecVerifyError(lib().ss_last_error().decode())
    return int(n)


def ss_spec_verify_attn(d: Dict[str, object], out: torch.Tensor, lse: Optional[torch.Tensor],
                        workspace: torch.Tensor, max_q_len: int = 0, reuse_plan: bool = False) -> None:
    """Enqueue verify attention for a device batch; `out`/`lse`/`workspace` are caller-owned device tensors."""
    kv, bt = _descriptors(d, max_q_len, SS_BATCH_REUSE_PLAN if reuse_plan else 0)
    _check(lib().ss_spec_verify_attn(ctypes.byref(kv), ctypes.byref(bt), _ptr(d["q"]), _DT[d["q_dtype"]],
                                     d["num_q_heads"], d["total_rows"], ctypes.c_float(d["sm_scale"]), _ptr(out),
                                     _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream()))


def alloc_attention_outputs(d: Dict[str, object], device="cuda:0", max_q_len: int = 0):
    """Allocate (out, lse, workspace) for a device batch.  `out` holds raw storage (int16 = bf16 bits)."""
    shape = (d["total_rows"], d["num_q_heads"], d["head_dim"])
    out = torch.empty(shape, dtype=torch.float32 if d["q_dtype"] == "f32" else torch.int16, device=device)
    lse = torch.empty(shape[:2], dtype=torch.float32, device=device)
    ws = torch.empty(max(ss_spec_verify_attn_workspace(d, max_q_len), 256), dtype=torch.uint8, device=device)
    return out, lse, ws


def ss_kv_append(d: Dict[str, object], max_q_len: int = 0) -> None:
    """Enqueue the append of `k_new`/`v_new` into the device batch's paged cache (written in place)."""
    kv, bt = _descriptors(d, max_q_len)
    _check(lib().ss_kv_append(ctypes.byref(kv), ctypes.byref(bt), _ptr(d["k_new"]), _ptr(d["v_new"]),
                              _DT[d["new_dtype"]], d["total_rows"], _stream()))


def ss_kv_compact(d: Dict[str, object], accepted_nodes: torch.Tensor, accepted_len: torch.Tensor,
                  max_q_len: int = 0) -> None:
    """Enqueue the move of every request's accepted tree path to the slots a chain would occupy (cache in place)."""
    kv, bt = _descriptors(d, max_q_len)
    _check(lib().ss_kv_compact(ctypes.byref(kv), ctypes.byref(bt), _ptr(accepted_nodes), _ptr(accepted_len),
                               d["total_rows"], _stream()))


def ss_kv_commit(q_indptr: torch.Tensor, accepted_len: torch.Tensor, kv_len: torch.Tensor) -> None:
    """Enqueue kv_len[b] <- kv_len[b] - k_b + accepted_len[b] on device int32 tensors (kv_len in place)."""
    _check(lib().ss_kv_commit(int(kv_len.numel()), _ptr(q_indptr), _ptr(accepted_len), _ptr(kv_len), _stream()))


def ss_depth_init() -> ss_depth_state:
    st = ss_depth_state()
    _check(lib().ss_depth_init(ctypes.byref(st)))
    return st


def ss_depth_update(state: ss_depth_state, accept_rate: float, load: float, throughput: float):
    """One controller step on the host; returns (d_star, b_micro, t_proj, k)."""
    d, b, t, k = ctypes.c_double(), ctypes.c_int32(), ctypes.c_double(), ctypes.c_int32()
    _check(lib().ss_depth_update(ctypes.byref(state), accept_rate, load, throughput, ctypes.byref(d), ctypes.byref(b),
                                 ctypes.byref(t), ctypes.byref(k)))
    return d.value, b.value, t.value, k.value


def ss_route_select(workers, q_max: float, alpha=None, tau: float = 0.0) -> int:
    """workers: sequence of (cache_hit, mem, queue_depth, load, stale).  Returns the chosen index."""
    arr = (ss_worker_metrics * len(workers))()
    for i, (c, m, d, l, st) in enumerate(workers):
        arr[i] = ss_worker_metrics(c, m, l, int(d), int(bool(st)))
    al = None if alpha is None else (ctypes.c_double * 4)(*alpha)
    out = ctypes.c_int32(-1)
    _check(lib().ss_route_select(arr, len(workers), al, tau, q_max, ctypes.byref(out)))
    return out.value


def ss_spec_accept_workspace(batch: int, total_rows: int, vocab: int) -> int:
    n = lib().ss_spec_accept_workspace(batch, total_rows, vocab)
    if n == 0 and batch > 0:
        raise SpecVerifyError(lib().ss_last_error().decode())
    return int(n)


def ss_spec_accept(d: Dict[str, object], accepted_len: torch.Tensor, out_tokens: torch.Tensor,
                   ratio_out: Optional[torch.Tensor], workspace: torch.Tensor, *, greedy: Optional[bool] = None,
                   per_request_temperature: bool = True, max_q_len: int = 0) -> None:
    g = d["greedy"] if greedy is None else int(greedy)
    temp = d["temperature"] if per_request_temperature else None
    t_scalar = 0.0 if per_request_temperature else float(d["temperature_scalar"])
    _check(lib().ss_spec_accept(d["batch"], d["vocab"], d["row_stride"], _DT[d["logit_dtype"]], d["total_rows"],
                                max_q_len, _ptr(d["q_indptr"]), _ptr(d["target_logits"]), _ptr(d["draft_logits"]),
                                _ptr(d["draft_tokens"]), _ptr(d["u_accept"]), _ptr(d["u_sample"]), _ptr(temp),
                                ctypes.c_float(t_scalar), g, _ptr(accepted_len), _ptr(out_tokens), _ptr(ratio_out),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def ss_spec_accept_static(d: Dict[str, object], accepted_len: torch.Tensor, out_tokens: torch.Tensor,
                          ratio_out: Optional[torch.Tensor], *, greedy: Optional[bool] = None,
                          per_request_temperature: bool = True, max_q_len: int = 0) -> None:
    """ss_spec_accept without a workspace argument: the library's static device array holds the partial results."""
    g = d["greedy"] if greedy is None else int(greedy)
    temp = d["temperature"] if per_request_temperature else None
    t_scalar = 0.0 if per_request_temperature else float(d["temperature_scalar"])
    _check(lib().ss_spec_accept_static(d["batch"], d["vocab"], d["row_stride"], _DT[d["logit_dtype"]], d["total_rows"],
                                       max_q_len, _ptr(d["q_indptr"]), _ptr(d["target_logits"]), _ptr(d["draft_logits"]),
                                       _ptr(d["draft_tokens"]), _ptr(d["u_accept"]), _ptr(d["u_sample"]), _ptr(temp),
                                       ctypes.c_float(t_scalar), g, _ptr(accepted_len), _ptr(out_tokens), _ptr(ratio_out),
                                       _stream()))


def ss_spec_accept_static_capacity() -> int:
    return int(lib().ss_spec_accept_static_capacity())


def ss_spec_accept_tree_greedy(d: Dict[str, object], accepted_len: torch.Tensor, out_tokens: torch.Tensor,
                               accepted_nodes: torch.Tensor, workspace: torch.Tensor, max_q_len: int = 0) -> None:
    _check(lib().ss_spec_accept_tree_greedy(d["batch"], d["vocab"], d["row_stride"], _DT[d["logit_dtype"]],
                                            d["total_rows"], max_q_len, _ptr(d["q_indptr"]), _ptr(d["tree_parent"]),
                                            _ptr(d["target_logits"]), _ptr(d["draft_tokens"]), _ptr(accepted_len),
                                            _ptr(out_tokens), _ptr(accepted_nodes), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream()))


def ss_spec_accept_tree_sample(d: Dict[str, object], accepted_len: torch.Tensor, out_tokens: torch.Tensor,
                               accepted_nodes: torch.Tensor, ratio_out: Optional[torch.Tensor], workspace: torch.Tensor,
                               max_q_len: int = 0) -> None:
    _check(lib().ss_spec_accept_tree_sample(d["batch"], d["vocab"], d["row_stride"], _DT[d["logit_dtype"]],
                                            d["total_rows"], max_q_len, _ptr(d["q_indptr"]), _ptr(d["tree_parent"]),
                                            _ptr(d["target_logits"]), _ptr(d["draft_logits"]), _ptr(d["draft_tokens"]),
                                            _ptr(d["u_accept"]), _ptr(d["u_sample"]), _ptr(d["temperature"]),
                                            ctypes.c_float(0.0), _ptr(accepted_len), _ptr(out_tokens),
                                            _ptr(accepted_nodes), _ptr(ratio_out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream()))


def tree_sample_workspace(d: Dict[str, object], device="cuda:0") -> torch.Tensor:
    n = lib().ss_spec_accept_tree_sample_workspace(d["batch"], d["total_rows"], d["vocab"])
    if n == 0 and d["batch"] > 0:
        raise SpecVerifyError(lib().ss_last_error().decode())
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


def alloc_accept_outputs(d: Dict[str, object], device="cuda:0"):
    B = d["batch"]
    acc = torch.full((B,), -77, dtype=torch.int32, device=device)
    toks = torch.full((B, SS_OUT_WIDTH), -77, dtype=torch.int32, device=device)
    ratio = torch.full((max(d["total_rows"] - B, 1),), float("nan"), dtype=torch.float32, device=device)
    ws = torch.empty(max(ss_spec_accept_workspace(B, d["total_rows"], d["vocab"]), 256), dtype=torch.uint8,
                     device=device)
    return acc, toks, ratio, ws


def bf16_bits_to_float(t: torch.Tensor) -> np.ndarray:
    """Raw int16 bf16 storage (device or host tensor) -> float64 numpy, exactly."""
    return t.cpu().view(torch.bfloat16).to(torch.float64).numpy()
