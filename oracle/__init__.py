"""ctypes front-end of the CPU oracle (``spec_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg, never by the product package.  It compiles the
C file with gcc on first use (or through ``build()``) and marshals numpy arrays;
all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spec_oracle.c")
_LIB = os.path.join(_HERE, "libspec_oracle.so")
_DT = {"f32": 0, "bf16": 1, "fp8": 2}
OUT_WIDTH = 21  # draft depth is at most 20 (the controller's d_max), so at most 21 tokens come out per request

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP only for the outer request loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_verify_attn.restype = ctypes.c_int
        lib.oracle_spec_accept.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_decode.restype = None
        lib.oracle_encode.restype = None
        lib.oracle_kv_append.restype = ctypes.c_int
        lib.oracle_kv_commit.restype = ctypes.c_int
        lib.oracle_tree_accept_greedy.restype = ctypes.c_int
        lib.oracle_kv_compact.restype = ctypes.c_int
        lib.oracle_tree_accept_sample.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def decode(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x)
    out = np.empty(x.shape, dtype=np.float64)
    _load().oracle_decode(_p(x), ctypes.c_int64(x.size), ctypes.c_int(_DT[dtype]), _p(out))
    return out


def verify_attn(inp: Dict[str, object], *, part_tokens: int = 0,
                requests: Optional[Sequence[int]] = None, threads: int = 0):
    """Run the attention oracle on a batch dict from ``synth.make_attention_inputs``.

    Returns (out[R,Hq,D] float64, lse[R,Hq] float64); rows of requests not in
    ``requests`` are NaN.  A ``tree_mask`` entry in the dict (uint32 per query row) makes the new
    tokens a draft tree; without it they are a chain.
    """
    lib = _load()
    R, Hq, D = inp["total_rows"], inp["num_q_heads"], inp["head_dim"]
    out = np.full((R, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((R, Hq), np.nan, dtype=np.float64)
    req = None if requests is None else np.ascontiguousarray(requests, dtype=np.int32)
    rc = lib.oracle_verify_attn(
        ctypes.c_int(inp["batch"]), ctypes.c_int(Hq), ctypes.c_int(inp["num_kv_heads"]),
        ctypes.c_int(D), ctypes.c_int(inp["block_size"]), ctypes.c_int(inp["max_blocks_per_seq"]),
        ctypes.c_int(_DT[inp["kv_dtype"]]), _p(inp["k_cache"]), _p(inp["v_cache"]),
        _p(inp["k_scale"]), _p(inp["v_scale"]), _p(inp["block_table"]), _p(inp["kv_len"]),
        _p(inp["q_indptr"]), _p(inp.get("tree_mask")), ctypes.c_int(_DT[inp["q_dtype"]]), _p(inp["q"]),
        ctypes.c_double(inp["sm_scale"]), ctypes.c_int(part_tokens), _p(req),
        ctypes.c_int(0 if req is None else len(req)), _p(out), _p(lse), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError(f"oracle_verify_attn rejected its arguments (code {rc})")
    return out, lse


def spec_accept(inp: Dict[str, object], *, greedy: Optional[bool] = None, tie_eps: float = 1e-5,
                threads: int = 0) -> Dict[str, np.ndarray]:
    """Run the acceptance oracle on a batch dict from ``synth.make_accept_inputs``."""
    lib = _load()
    B, R = inp["batch"], inp["total_rows"]
    Rd = R - B
    g = inp["greedy"] if greedy is None else int(greedy)
    accepted = np.full(B, -99, dtype=np.int32)
    toks = np.full((B, OUT_WIDTH), -99, dtype=np.int32)
    ratio = np.full(max(Rd, 1), np.nan, dtype=np.float64)
    near = np.zeros(max(Rd, 1), dtype=np.int32)
    ylo = np.full(B, -1, dtype=np.int32)
    yhi = np.full(B, -1, dtype=np.int32)
    rsum = np.full(B, np.nan, dtype=np.float64)
    rc = lib.oracle_spec_accept(
        ctypes.c_int(B), ctypes.c_int(inp["vocab"]), ctypes.c_int64(inp["row_stride"]),
        ctypes.c_int(_DT[inp["logit_dtype"]]), _p(inp["q_indptr"]), _p(inp["target_logits"]),
        _p(inp["draft_logits"]), _p(inp["draft_tokens"]), _p(inp["u_accept"]), _p(inp["u_sample"]),
        _p(inp["temperature"]), ctypes.c_int(g), ctypes.c_int(OUT_WIDTH), ctypes.c_double(tie_eps),
        _p(accepted), _p(toks), _p(ratio), _p(near), _p(ylo), _p(yhi), _p(rsum),
        ctypes.c_int(threads))
    if rc != 0:
        raise ValueError(f"oracle_spec_accept rejected its arguments (code {rc})")
    return dict(accepted_len=accepted, out_tokens=toks, ratio=ratio[:Rd], near_tie=near[:Rd],
                y_lo=ylo, y_hi=yhi, resid_sum=rsum)


def tree_accept_greedy(inp: Dict[str, object]) -> Dict[str, np.ndarray]:
    """Greedy acceptance walk over the draft trees of a batch dict from ``synth.make_tree_accept_inputs``."""
    B = inp["batch"]
    accepted = np.full(B, -99, dtype=np.int32)
    toks = np.full((B, OUT_WIDTH), -99, dtype=np.int32)
    nodes = np.full((B, OUT_WIDTH - 1), -99, dtype=np.int32)
    rc = _load().oracle_tree_accept_greedy(
        ctypes.c_int(B), ctypes.c_int(inp["vocab"]), ctypes.c_int64(inp["row_stride"]),
        ctypes.c_int(_DT[inp["logit_dtype"]]), _p(inp["q_indptr"]), _p(inp["tree_parent"]),
        _p(inp["target_logits"]), _p(inp["draft_tokens"]), ctypes.c_int(OUT_WIDTH), _p(accepted), _p(toks), _p(nodes))
    if rc != 0:
        raise ValueError(f"oracle_tree_accept_greedy rejected its arguments (code {rc})")
    return dict(accepted_len=accepted, out_tokens=toks, accepted_nodes=nodes)


def tree_accept_sample(inp: Dict[str, object], tie_eps: float = 1e-5) -> Dict[str, np.ndarray]:
    """Sampled acceptance walk over the draft trees of a batch dict from ``synth.make_tree_accept_inputs``."""
    B, Rd = inp["batch"], inp["total_rows"] - inp["batch"]
    accepted = np.full(B, -99, dtype=np.int32)
    toks = np.full((B, OUT_WIDTH), -99, dtype=np.int32)
    nodes = np.full((B, OUT_WIDTH - 1), -99, dtype=np.int32)
    ratio = np.full(max(Rd, 1), np.nan, dtype=np.float64)
    near = np.zeros(max(Rd, 1), dtype=np.int32)
    rc = _load().oracle_tree_accept_sample(
        ctypes.c_int(B), ctypes.c_int(inp["vocab"]), ctypes.c_int64(inp["row_stride"]),
        ctypes.c_int(_DT[inp["logit_dtype"]]), _p(inp["q_indptr"]), _p(inp["tree_parent"]),
        _p(inp["target_logits"]), _p(inp["draft_logits"]), _p(inp["draft_tokens"]), _p(inp["u_accept"]),
        _p(inp["u_sample"]), _p(inp["temperature"]), ctypes.c_int(OUT_WIDTH), ctypes.c_double(tie_eps),
        _p(accepted), _p(toks), _p(nodes), _p(ratio), _p(near))
    if rc != 0:
        raise ValueError(f"oracle_tree_accept_sample rejected its arguments (code {rc})")
    return dict(accepted_len=accepted, out_tokens=toks, accepted_nodes=nodes, ratio=ratio[:Rd], near_tie=near[:Rd])


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 -> bfloat16 bits (uint16) or e4m3fn bytes (uint8, |x| <= 448), nearest, ties to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16 if dtype == "bf16" else np.uint8)
    _load().oracle_encode(_p(x), ctypes.c_int64(x.size), ctypes.c_int(_DT[dtype]), _p(out))
    return out


def kv_append(inp: Dict[str, object]) -> None:
    """Write the new tokens' K/V of a batch dict from ``synth.make_append_inputs`` into its cache, in place."""
    rc = _load().oracle_kv_append(
        ctypes.c_int(inp["batch"]), ctypes.c_int(inp["num_kv_heads"]), ctypes.c_int(inp["head_dim"]),
        ctypes.c_int(inp["block_size"]), ctypes.c_int(inp["max_blocks_per_seq"]), ctypes.c_int(_DT[inp["kv_dtype"]]),
        _p(inp["k_cache"]), _p(inp["v_cache"]), _p(inp["k_scale"]), _p(inp["v_scale"]), _p(inp["block_table"]),
        _p(inp["kv_len"]), _p(inp["q_indptr"]), ctypes.c_int(_DT[inp["new_dtype"]]), _p(inp["k_new"]), _p(inp["v_new"]))
    if rc != 0:
        raise ValueError(f"oracle_kv_append rejected its arguments (code {rc})")


def kv_compact(inp: Dict[str, object], accepted_nodes: np.ndarray, accepted_len: np.ndarray) -> None:
    """Move the accepted tree path of every request to the slots a chain would occupy, in place."""
    nodes = np.ascontiguousarray(accepted_nodes, dtype=np.int32)
    rc = _load().oracle_kv_compact(
        ctypes.c_int(inp["batch"]), ctypes.c_int(inp["num_kv_heads"]), ctypes.c_int(inp["head_dim"]),
        ctypes.c_int(inp["block_size"]), ctypes.c_int(inp["max_blocks_per_seq"]), ctypes.c_int(_DT[inp["kv_dtype"]]),
        _p(inp["k_cache"]), _p(inp["v_cache"]), _p(inp["k_scale"]), _p(inp["v_scale"]), _p(inp["block_table"]),
        _p(inp["kv_len"]), _p(inp["q_indptr"]), _p(nodes), ctypes.c_int(nodes.shape[1]),
        _p(np.ascontiguousarray(accepted_len, dtype=np.int32)))
    if rc != 0:
        raise ValueError(f"oracle_kv_compact rejected its arguments (code {rc})")


def kv_commit(q_indptr: np.ndarray, accepted_len: np.ndarray, kv_len: np.ndarray) -> np.ndarray:
    """Valid cache length of every request after acceptance (a new array)."""
    out = np.ascontiguousarray(kv_len, dtype=np.int32).copy()
    rc = _load().oracle_kv_commit(ctypes.c_int(len(out)), _p(np.ascontiguousarray(q_indptr, dtype=np.int32)),
                                  _p(np.ascontiguousarray(accepted_len, dtype=np.int32)), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_kv_commit rejected its arguments (code {rc})")
    return out
