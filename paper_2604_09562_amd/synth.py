"""Seeded synthetic inputs for the speculative-verification step.

This module only *draws* inputs (lengths, depths, Q/K/V values, block tables,
logits, draft tokens, uniforms) and rounds them once to their storage format.
It contains none of the verification arithmetic: both the CPU oracle and the
HIP library consume the exact bytes produced here, each decoding them with its
own code.

The paper (Section 3.5, Alg. 4 and Eq. 13) only fixes that every request
carries its own speculation depth; the decode worker then verifies that many
draft tokens in one target pass (Section 2.2) over a paged KV cache
(Section 2.4) that already holds the prefill KV plus everything decoded so far
(Section 3.4, Eq. 7).  The shapes below stand in for the paper's decode
workloads (its datasets and model weights are not used).

Storage formats
---------------
* ``f32``  : numpy float32
* ``bf16`` : numpy uint16 holding the upper 16 bits of the float32 (RNE)
* ``fp8``  : numpy uint8 holding OCP e4m3fn bytes (RNE, saturating at +-448);
             real value = decode(byte) * scale[block, kv_head]

Paged KV layout: ``[num_blocks][num_kv_heads][block_size=16][head_dim]``.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Sequence, Tuple

import numpy as np
import torch

BLOCK_SIZE = 16
KMAX = 20  # largest draft depth a request may carry (the controller's d_max; the five workloads stay within 8)

_SEED_BASE = 9_562_000


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    name: str
    index: int
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    kv_dtype: str            # 'f32' | 'bf16' | 'fp8'
    q_dtype: str             # 'f32' | 'bf16'
    ctx: Tuple               # ('fixed', [..]) | ('uniform', lo, hi) | ('loguniform', lo, hi)
    depth: Tuple             # ('fixed', k) | ('uniform', lo, hi)
    vocab: int
    logit_dtype: str         # 'f32' | 'bf16'
    sigma_target: float
    spike: float             # added to one seeded token per target row (0 = none)
    sigma_draft: Tuple       # ('fixed', s) | ('uniform', lo, hi) per request
    temperature: float

    def scaled(self, **kw) -> "VerifyConfig":
        """Same recipe at a different size (used by CPU tests and the bounded CPU baseline)."""
        return dataclasses.replace(self, **kw)


CONFIGS: Sequence[VerifyConfig] = (
    VerifyConfig("tiny_f32", 0, 4, 8, 2, 64, "f32", "f32",
                 ("fixed", (64, 128, 256, 512)), ("fixed", 4),
                 1024, "f32", 2.0, 0.0, ("fixed", 0.5), 1.0),
    VerifyConfig("llama3_8b_b64", 1, 64, 32, 8, 128, "bf16", "bf16",
                 ("uniform", 256, 4096), ("fixed", 4),
                 128256, "bf16", 3.0, 8.0, ("fixed", 1.0), 0.8),
    VerifyConfig("ragged_b128", 2, 128, 32, 8, 128, "bf16", "bf16",
                 ("loguniform", 128, 16384), ("uniform", 0, 8),
                 128256, "bf16", 3.0, 0.0, ("uniform", 0.3, 3.0), 1.0),
    VerifyConfig("long_b16", 3, 16, 32, 8, 128, "bf16", "bf16",
                 ("uniform", 16384, 65536), ("fixed", 6),
                 128256, "bf16", 3.0, 0.0, ("fixed", 1.0), 1.0),
    VerifyConfig("llama70b_fp8_b96", 4, 96, 64, 8, 128, "fp8", "bf16",
                 ("uniform", 512, 8192), ("uniform", 2, 8),
                 152064, "bf16", 3.0, 0.0, ("fixed", 0.8), 0.7),
)


def config_by_name(name: str) -> VerifyConfig:
    for c in CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)


def _rng(cfg: VerifyConfig, seed: int, stream: int) -> np.random.Generator:
    # streams: 0 lengths/depths, 1 Q, 2 KV, 3 block permutation, 4 logits,
    #          5 uniforms, 6 draft-token sampling, 7 fp8 scales, 8 per-request draft sigma
    return np.random.Generator(np.random.PCG64(_SEED_BASE + 1000 * seed + 10 * cfg.index + stream))


# ----------------------------------------------------------------------------
# storage rounding (done once; the rounded bytes are THE input)
# ----------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def to_fp8_bytes(x: np.ndarray) -> np.ndarray:
    """Encode already-scaled values as e4m3fn, saturating (never producing the NaN byte)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp_(-448.0, 448.0)
    b = t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert not np.any((b & 0x7F) == 0x7F), "fp8 encoder produced a NaN byte"
    return b


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return to_bf16_bits(x)
    raise ValueError(dtype)


def draw_lengths(cfg: VerifyConfig, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-request kv_len (valid cache positions, including this step's k+1 new tokens) and depth k."""
    rng = _rng(cfg, seed, 0)
    B = cfg.batch
    kind = cfg.ctx[0]
    if kind == "fixed":
        vals = np.asarray(cfg.ctx[1], dtype=np.int64)
        kv_len = vals[np.arange(B) % len(vals)]
    elif kind == "uniform":
        kv_len = rng.integers(cfg.ctx[1], cfg.ctx[2] + 1, size=B)
    elif kind == "loguniform":
        u = rng.uniform(math.log(cfg.ctx[1]), math.log(cfg.ctx[2]), size=B)
        kv_len = np.rint(np.exp(u)).astype(np.int64)
    else:
        raise ValueError(kind)
    if cfg.depth[0] == "fixed":
        k = np.full(B, cfg.depth[1], dtype=np.int64)
    else:
        k = rng.integers(cfg.depth[1], cfg.depth[2] + 1, size=B)
    assert k.min() >= 0 and k.max() <= KMAX
    kv_len = np.maximum(kv_len, k + 1)
    return kv_len.astype(np.int32), k.astype(np.int32)


def make_attention_inputs(cfg: VerifyConfig, seed: int = 0, *,
                          nan_tail: bool = False,
                          kv_len: Optional[np.ndarray] = None,
                          depth: Optional[np.ndarray] = None,
                          tree: bool = False) -> Dict[str, object]:
    """Draw one batch for spec_verify_attn.

    Returns a dict of numpy arrays in storage format plus the scalar shape
    fields.  Slots past kv_len in a request's last block hold large finite
    garbage (NaN bytes when ``nan_tail``), pool blocks no request references
    hold NaN bytes, and block-table padding is -1: real caches look like that.
    With ``tree`` the new tokens of every request form a random draft tree
    (``tree_parent``, ``tree_mask``; see ``draw_draft_trees``) instead of a chain.
    """
    if kv_len is None or depth is None:
        kv_len_d, depth_d = draw_lengths(cfg, seed)
        kv_len = kv_len_d if kv_len is None else np.asarray(kv_len, dtype=np.int32)
        depth = depth_d if depth is None else np.asarray(depth, dtype=np.int32)
    B = len(kv_len)
    Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
    q_len = depth.astype(np.int64) + 1
    q_indptr = np.zeros(B + 1, dtype=np.int32)
    q_indptr[1:] = np.cumsum(q_len)
    R = int(q_indptr[-1])

    nblk = (kv_len.astype(np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE
    used = int(nblk.sum())
    num_blocks = int(math.ceil(1.1 * used)) + 1
    max_blocks = int(nblk.max())
    perm = _rng(cfg, seed, 3).permutation(num_blocks)[:used].astype(np.int32)
    block_table = np.full((B, max_blocks), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        n = int(nblk[b])
        block_table[b, :n] = perm[off:off + n]
        off += n

    rq = _rng(cfg, seed, 1)
    q = store(rq.standard_normal((R, Hq, D), dtype=np.float32), cfg.q_dtype)

    rkv = _rng(cfg, seed, 2)
    rsc = _rng(cfg, seed, 7)
    tile = (Hkv, BLOCK_SIZE, D)
    if cfg.kv_dtype == "f32":
        np_dtype, nan_fill, big = np.float32, np.float32(np.nan), np.float32(1.0e4)
    elif cfg.kv_dtype == "bf16":
        np_dtype, nan_fill, big = np.uint16, np.uint16(0x7FC0), to_bf16_bits(np.array([1.0e4]))[0]
    elif cfg.kv_dtype == "fp8":
        np_dtype, nan_fill, big = np.uint8, np.uint8(0x7F), np.uint8(0x7E)  # 0x7E = +448
    else:
        raise ValueError(cfg.kv_dtype)
    k_cache = np.full((num_blocks,) + tile, nan_fill, dtype=np_dtype)
    v_cache = np.full((num_blocks,) + tile, nan_fill, dtype=np_dtype)
    k_scale = v_scale = None
    if cfg.kv_dtype == "fp8":
        k_scale = rsc.uniform(0.01, 0.1, size=(num_blocks, Hkv)).astype(np.float32)
        v_scale = rsc.uniform(0.01, 0.1, size=(num_blocks, Hkv)).astype(np.float32)

    # fill referenced blocks, a chunk of physical blocks at a time (bounded host memory)
    CH = 4096
    for lo in range(0, used, CH):
        ids = perm[lo:lo + CH]
        n = len(ids)
        for cache, scale in ((k_cache, k_scale), (v_cache, v_scale)):
            x = rkv.standard_normal((n,) + tile, dtype=np.float32)
            if cfg.kv_dtype == "fp8":
                cache[ids] = to_fp8_bytes(x / scale[ids][:, :, None, None])
            elif cfg.kv_dtype == "bf16":
                cache[ids] = to_bf16_bits(x)
            else:
                cache[ids] = x
    # garbage in the unused slots of each request's last block
    tail_val = nan_fill if nan_tail else big
    for b in range(B):
        r = int(kv_len[b]) % BLOCK_SIZE
        if r:
            last = block_table[b, int(nblk[b]) - 1]
            k_cache[last, :, r:, :] = tail_val
            v_cache[last, :, r:, :] = tail_val

    out = dict(
        batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, block_size=BLOCK_SIZE,
        num_blocks=num_blocks, max_blocks_per_seq=max_blocks, total_rows=R,
        kv_dtype=cfg.kv_dtype, q_dtype=cfg.q_dtype,
        kv_len=kv_len.astype(np.int32), depth=depth.astype(np.int32), q_indptr=q_indptr,
        block_table=block_table, k_cache=k_cache, v_cache=v_cache,
        k_scale=k_scale, v_scale=v_scale, q=q, sm_scale=float(1.0 / math.sqrt(D)),
    )
    if tree:
        out["tree_parent"], out["tree_mask"] = draw_draft_trees(q_indptr, _rng(cfg, seed, 10))
    return out


def draw_draft_trees(q_indptr: np.ndarray, rng: np.random.Generator):
    """Random draft trees over the query rows of a batch.

    Row 0 of a request is the tree's root (the last accepted token); row i > 0 is a draft node whose
    parent is drawn uniformly from rows 0..i-1 of the same request, so parents precede children, as
    in a tree stored level by level or in depth-first order.  Returns ``tree_parent`` (int32 per
    row, index within the request, -1 for the root) and ``tree_mask`` (uint32 per row: bit j set
    iff row j of the request is the row itself or one of its ancestors).
    """
    R = int(q_indptr[-1])
    parent = np.full(R, -1, dtype=np.int32)
    mask = np.zeros(R, dtype=np.uint32)
    for b in range(len(q_indptr) - 1):
        r0, n = int(q_indptr[b]), int(q_indptr[b + 1] - q_indptr[b])
        mask[r0] = 1
        for i in range(1, n):
            p = int(rng.integers(0, i))
            parent[r0 + i] = p
            mask[r0 + i] = mask[r0 + p] | np.uint32(1 << i)
    return parent, mask


def make_append_inputs(cfg: VerifyConfig, seed: int = 0, **kw) -> Dict[str, object]:
    """A batch for kv_append: the attention batch with the new tokens' cache slots poisoned, plus
    the new keys/values ``k_new``/``v_new`` [total_rows][kv heads][head_dim] (N(0,1), float32 for a
    float32 cache, bfloat16 bits otherwise) that the append has to write there.  For e4m3 caches the
    scales of the blocks this step starts are poisoned too (the append must set them)."""
    inp = make_attention_inputs(cfg, seed, **kw)
    B, Hkv, D, R = inp["batch"], inp["num_kv_heads"], inp["head_dim"], inp["total_rows"]
    rng = _rng(cfg, seed, 9)
    new_dtype = "f32" if cfg.kv_dtype == "f32" else "bf16"
    inp["new_dtype"] = new_dtype
    inp["k_new"] = store(rng.standard_normal((R, Hkv, D), dtype=np.float32), new_dtype)
    inp["v_new"] = store(rng.standard_normal((R, Hkv, D), dtype=np.float32), new_dtype)
    poison = {"f32": np.float32(np.nan), "bf16": np.uint16(0x7FC0), "fp8": np.uint8(0x7F)}[cfg.kv_dtype]
    for b in range(B):
        q_len = int(inp["q_indptr"][b + 1] - inp["q_indptr"][b])
        L = int(inp["kv_len"][b])
        for pos in range(L - q_len, L):
            phys = inp["block_table"][b, pos // BLOCK_SIZE]
            inp["k_cache"][phys, :, pos % BLOCK_SIZE, :] = poison
            inp["v_cache"][phys, :, pos % BLOCK_SIZE, :] = poison
            if cfg.kv_dtype == "fp8" and pos % BLOCK_SIZE == 0:
                inp["k_scale"][phys, :] = np.nan
                inp["v_scale"][phys, :] = np.nan
    return inp


def _sample_rows_inverse_cdf(logits: np.ndarray, T: np.ndarray, u: np.ndarray) -> np.ndarray:
    """Draw one token per row from softmax(logits/T) (draft-model sampling: workload, not verification)."""
    out = np.empty(len(logits), dtype=np.int32)
    for r in range(len(logits)):
        z = logits[r].astype(np.float64) / float(T[r])
        w = np.exp(z - z.max())
        c = np.cumsum(w)
        out[r] = min(int(np.searchsorted(c, u[r] * c[-1], side="right")), logits.shape[1] - 1)
    return out


def make_accept_inputs(cfg: VerifyConfig, seed: int = 0, *, depth: Optional[np.ndarray] = None,
                       greedy: bool = False, row_pad: int = 0) -> Dict[str, object]:
    """Draw one batch for spec_accept.

    Target rows: q_indptr layout (request b owns rows q_indptr[b]..q_indptr[b+1]-1,
    row i judges draft i, the last row is the bonus distribution).  Draft rows:
    request b's k_b rows start at q_indptr[b]-b.  Draft tokens are drawn from the
    draft distribution itself (sampling mode) or are its argmax (greedy mode), as
    a draft model would produce them.
    """
    if depth is None:
        _, depth = draw_lengths(cfg, seed)
    depth = np.asarray(depth, dtype=np.int32)
    B, V = len(depth), cfg.vocab
    q_indptr = np.zeros(B + 1, dtype=np.int32)
    q_indptr[1:] = np.cumsum(depth.astype(np.int64) + 1)
    R = int(q_indptr[-1])
    Rd = R - B
    stride = V + row_pad

    rl = _rng(cfg, seed, 4)
    if cfg.sigma_draft[0] == "fixed":
        sig_d = np.full(B, cfg.sigma_draft[1], dtype=np.float64)
    else:
        sig_d = _rng(cfg, seed, 8).uniform(cfg.sigma_draft[1], cfg.sigma_draft[2], size=B)

    tgt = np.empty((R, stride), dtype=np.float32)
    drf = np.empty((max(Rd, 1), stride), dtype=np.float32)
    pad_val = np.float32(3.0e4)  # padding past the vocabulary must never be read
    tgt[:, V:] = pad_val
    drf[:, V:] = pad_val
    for b in range(B):
        for i in range(int(depth[b]) + 1):
            row = rl.standard_normal(V, dtype=np.float32) * np.float32(cfg.sigma_target)
            if cfg.spike:
                row[int(rl.integers(0, V))] += np.float32(cfg.spike)
            tgt[q_indptr[b] + i, :V] = row
            if i < depth[b]:
                noise = rl.standard_normal(V, dtype=np.float32) * np.float32(sig_d[b])
                drf[q_indptr[b] - b + i, :V] = row + noise
    drf = drf[:Rd] if Rd > 0 else drf[:0]
    tgt_s = store(tgt, cfg.logit_dtype)
    drf_s = store(drf, cfg.logit_dtype)

    temperature = np.full(B, cfg.temperature, dtype=np.float32)
    ru = _rng(cfg, seed, 5)
    u_accept = ru.random(Rd, dtype=np.float32)
    u_sample = ru.random(B, dtype=np.float32)

    # draft tokens come from the *stored* (rounded) draft logits
    drf_val = decode_storage(drf_s, cfg.logit_dtype)[:, :V] if Rd > 0 else np.zeros((0, V), np.float32)
    row_T = np.repeat(temperature, depth)
    if greedy:
        draft_tokens = np.argmax(drf_val, axis=1).astype(np.int32)
    else:
        draft_tokens = _sample_rows_inverse_cdf(drf_val, row_T, _rng(cfg, seed, 6).random(Rd))
    return dict(
        batch=B, vocab=V, row_stride=stride, logit_dtype=cfg.logit_dtype, total_rows=R,
        depth=depth, q_indptr=q_indptr, target_logits=tgt_s, draft_logits=drf_s,
        draft_tokens=draft_tokens, u_accept=u_accept, u_sample=u_sample,
        temperature=temperature, greedy=int(greedy), sigma_draft=sig_d,
    )


def make_tree_accept_inputs(cfg: VerifyConfig, seed: int = 0, *, depth: Optional[np.ndarray] = None,
                            hit: float = 0.6, row_pad: int = 0) -> Dict[str, object]:
    """A batch for greedy acceptance over draft trees.

    Target logits, layout and sizes are those of ``make_accept_inputs``; the drafts of a request
    form the random tree of ``draw_draft_trees`` (the same tree ``make_attention_inputs(tree=True)``
    draws for these depths and seed).  A draft node carries, with probability ``hit``, the token
    greedy decoding would emit after its parent (the lowest-index maximum of the parent's stored
    target row), as a good draft model's candidates do; otherwise, with probability 0.15, a copy of
    an earlier sibling's token, and else a uniformly random token.
    """
    inp = make_accept_inputs(cfg, seed, depth=depth, greedy=True, row_pad=row_pad)
    q_indptr, V = inp["q_indptr"], inp["vocab"]
    r = _rng(cfg, seed, 11)
    parent, mask = draw_draft_trees(q_indptr, _rng(cfg, seed, 10))
    tgt_val = decode_storage(inp["target_logits"], cfg.logit_dtype)[:, :V]
    best = np.argmax(tgt_val, axis=1)
    tokens = np.zeros(len(inp["draft_tokens"]), dtype=np.int32)
    for b in range(inp["batch"]):
        r0, n = int(q_indptr[b]), int(q_indptr[b + 1] - q_indptr[b])
        node_tok = [-1] * n
        for i in range(1, n):
            p = int(parent[r0 + i])
            sibs = [node_tok[j] for j in range(1, i) if parent[r0 + j] == p]
            u = r.random()
            if u < hit:
                node_tok[i] = int(best[r0 + p])
            elif u < hit + 0.15 and sibs:
                node_tok[i] = sibs[int(r.integers(0, len(sibs)))]
            else:
                node_tok[i] = int(r.integers(0, V))
            tokens[r0 - b + i - 1] = node_tok[i]
    inp["draft_tokens"] = tokens
    inp["tree_parent"], inp["tree_mask"] = parent, mask
    return inp


def make_tree_sample_inputs(cfg: VerifyConfig, seed: int = 0, *, depth: Optional[np.ndarray] = None,
                            row_pad: int = 0) -> Dict[str, object]:
    """A batch for sampled acceptance over draft trees.

    Target logits, uniforms, temperatures and sizes are those of ``make_accept_inputs``; the drafts of a
    request form the random tree of ``draw_draft_trees``.  The children of a node are drawn, as a draft
    model would, from one proposal: the node's target row plus N(0, sigma_draft) noise (one noise
    vector per parent), rounded to the logit dtype; draft row i-1 holds the proposal node i was drawn
    from, so siblings carry equal rows.
    """
    inp = make_accept_inputs(cfg, seed, depth=depth, row_pad=row_pad)
    q_indptr, V, stride = inp["q_indptr"], inp["vocab"], inp["row_stride"]
    B = inp["batch"]
    parent, mask = draw_draft_trees(q_indptr, _rng(cfg, seed, 10))
    rn = _rng(cfg, seed, 12)
    tgt = decode_storage(inp["target_logits"], cfg.logit_dtype)
    Rd = inp["total_rows"] - B
    drf = np.empty((max(Rd, 1), stride), dtype=np.float32)
    drf[:, V:] = np.float32(3.0e4)
    for b in range(B):
        r0, n = int(q_indptr[b]), int(q_indptr[b + 1] - q_indptr[b])
        proposal = {}
        for i in range(1, n):
            p = int(parent[r0 + i])
            if p not in proposal:
                noise = rn.standard_normal(V, dtype=np.float32) * np.float32(inp["sigma_draft"][b])
                proposal[p] = tgt[r0 + p, :V] + noise
            drf[r0 - b + i - 1, :V] = proposal[p]
    drf = drf[:Rd] if Rd > 0 else drf[:0]
    drf_s = store(drf, cfg.logit_dtype)
    drf_val = decode_storage(drf_s, cfg.logit_dtype)[:, :V] if Rd > 0 else np.zeros((0, V), np.float32)
    row_T = np.repeat(inp["temperature"], inp["depth"])
    inp["draft_logits"] = drf_s
    inp["draft_tokens"] = _sample_rows_inverse_cdf(drf_val, row_T, _rng(cfg, seed, 6).random(Rd))
    inp["tree_parent"], inp["tree_mask"] = parent, mask
    return inp


def decode_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Storage -> float32 via torch (generator-side helper for drawing draft tokens and for tests)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    if dtype == "fp8":
        return torch.from_numpy(x).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    raise ValueError(dtype)


def kv_bytes_algorithmic(inp: Dict[str, object]) -> int:
    """Bytes of K and V (plus fp8 scales) that one verify pass must read: the roofline numerator."""
    esz = {"f32": 4, "bf16": 2, "fp8": 1}[inp["kv_dtype"]]
    tokens = int(np.asarray(inp["kv_len"], dtype=np.int64).sum())
    n = tokens * inp["num_kv_heads"] * inp["head_dim"] * 2 * esz
    if inp["kv_dtype"] == "fp8":
        blocks = int(((np.asarray(inp["kv_len"], dtype=np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE).sum())
        n += blocks * inp["num_kv_heads"] * 2 * 4
    return n
