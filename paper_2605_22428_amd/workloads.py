"""Seeded synthetic inputs for the MultiWrite dispatch / AllGather hot path.

This module only *draws inputs*: router top-k expert ids, payload rows and
AllGather shards for every simulated rank.  It holds none of the method's
arithmetic (no bitmaps, no grouping, no packing, no receive-side layout) so
that the CPU oracle and the HIP path can both be fed from it without sharing
anything else.  It imports neither of them.

All randomness comes from a counter-based generator written out here
(splitmix64 finaliser applied to key and counter), so a value depends only on
(seed, workload, peer, token, column) and rows can be generated lazily in any
order.  The workloads stand in for the MoE dispatch the paper evaluates
(Section 6.1: 64 experts, top-8, batches of 64..2k tokens) scaled to the
DeepSeek-V3 shapes this build is measured on; no dataset or trained weights
are involved.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 260522428

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


# --------------------------------------------------------------------------
# counter-based generator
# --------------------------------------------------------------------------
def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wraps modulo 2**64)."""
    z = (z + _GOLD).astype(_U64, copy=False)
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def _key(*parts: int) -> np.uint64:
    """Fold small non-negative integers into one 64-bit stream key."""
    k = np.array([0x243F6A8885A308D3], dtype=_U64)
    for p in parts:
        k = _mix(k ^ np.array([int(p) & 0xFFFFFFFFFFFFFFFF], dtype=_U64))
    return k[0]


def _bits(key: np.uint64, counters: np.ndarray) -> np.ndarray:
    """64 random bits per counter for the stream `key`."""
    c = np.asarray(counters, dtype=_U64)
    return _mix(_mix(c ^ key) + key)


def _uniform(key: np.uint64, counters: np.ndarray) -> np.ndarray:
    """Uniform deviates in the open interval (0, 1), float64."""
    b = _bits(key, counters) >> _U64(11)
    return (b.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal(key: np.uint64, n: int) -> np.ndarray:
    """n standard normal deviates, float64 (Box-Muller: uniforms 2i and 2i+1
    give elements 2i (cosine branch) and 2i+1 (sine branch))."""
    m = (n + 1) // 2
    i2 = np.arange(m, dtype=_U64) * _U64(2)
    r = np.sqrt(-2.0 * np.log(_uniform(key, i2)))
    ang = (2.0 * np.pi) * _uniform(key, i2 + _U64(1))
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    return out[:n]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    b = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (b >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class DispatchWorkload:
    """One dispatch configuration: every simulated rank draws `n_tokens`
    tokens the same way from its own stream."""
    name: str
    wid: int                 # stream id folded into every key
    n_ranks: int             # R
    n_experts: int           # E, contiguous map e -> e // (E / R)
    top_k: int               # K
    n_tokens: int            # T per rank
    hidden: int              # H elements per token
    row_format: str          # "bf16" | "fp8"
    routing: str             # "uniform" | "dsv3" | "zipf"
    n_nodes: int = 1         # dsv3: ranks are split evenly over nodes
    max_nodes: int = 1       # dsv3: a token's experts span at most this many
    zipf_s: float = 1.1
    my_rank: int = 0

    @property
    def experts_per_rank(self) -> int:
        return self.n_experts // self.n_ranks

    @property
    def row_bytes(self) -> int:
        if self.row_format == "bf16":
            return 2 * self.hidden
        return self.hidden + 4 * (self.hidden // 128)


@dataclass(frozen=True)
class AllGatherWorkload:
    name: str
    wid: int
    n_ranks: int
    shard_elems: int         # bf16 elements per rank
    my_rank: int = 0

    @property
    def shard_bytes(self) -> int:
        return 2 * self.shard_elems


C0 = DispatchWorkload("C0_tiny", 0, 8, 16, 2, 128, 256, "bf16", "uniform")
C1 = DispatchWorkload("C1_dsv3_bf16", 1, 64, 256, 8, 4096, 7168, "bf16", "dsv3",
                      n_nodes=8, max_nodes=4)
# C2 shares C1's routing stream (same wid): it is C1 with an fp8 payload.
C2 = DispatchWorkload("C2_dsv3_fp8", 1, 64, 256, 8, 4096, 7168, "fp8", "dsv3",
                      n_nodes=8, max_nodes=4)
C3 = DispatchWorkload("C3_ep256_zipf", 3, 256, 256, 8, 8192, 7168, "bf16", "zipf")
C4 = AllGatherWorkload("C4_allgather", 4, 128, 1 << 20)

DISPATCH: Dict[str, DispatchWorkload] = {"C0": C0, "C1": C1, "C2": C2, "C3": C3}


def scaled(w: DispatchWorkload, *, n_tokens: Optional[int] = None,
           hidden: Optional[int] = None, my_rank: Optional[int] = None) -> DispatchWorkload:
    """Same routing structure with fewer tokens / a narrower row (for cases
    the CPU oracle has to finish in seconds)."""
    kw = {}
    if n_tokens is not None:
        kw["n_tokens"] = n_tokens
    if hidden is not None:
        kw["hidden"] = hidden
    if my_rank is not None:
        kw["my_rank"] = my_rank
    return replace(w, **kw)


def expert_to_rank(w: DispatchWorkload) -> np.ndarray:
    """Contiguous placement: expert e lives on rank e // (E / R)."""
    return (np.arange(w.n_experts, dtype=np.int32) // w.experts_per_rank).astype(np.int32)


def zipf_order(w: DispatchWorkload, seed: int) -> np.ndarray:
    """Seed-derived permutation: order[i] = expert id at popularity position i
    (position 0 is the hottest).  Shared by all peers of one run."""
    k = _key(seed, w.wid, 0xA11)
    return np.argsort(_bits(k, np.arange(w.n_experts)), kind="stable").astype(np.int32)


def zipf_median_rank(w: DispatchWorkload, seed: int) -> int:
    """Rank hosting the expert at the median popularity position (E / 2,
    counted from 1)."""
    e = int(zipf_order(w, seed)[w.n_experts // 2 - 1])
    return int(expert_to_rank(w)[e])


def zipf_hottest_rank(w: DispatchWorkload, seed: int) -> int:
    e = int(zipf_order(w, seed)[0])
    return int(expert_to_rank(w)[e])


# --------------------------------------------------------------------------
# router draws
# --------------------------------------------------------------------------
def _top_desc(score: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries per row, in descending score order,
    ties to the lower index."""
    n = score.shape[1]
    if k >= n:
        return np.argsort(-score, axis=1, kind="stable")[:, :k]
    part = np.argpartition(-score, k - 1, axis=1)[:, :k]
    part.sort(axis=1)                                   # ascending id so ties keep id order
    sub = np.take_along_axis(score, part, axis=1)
    order = np.argsort(-sub, axis=1, kind="stable")
    return np.take_along_axis(part, order, axis=1)


def topk_ids(w: DispatchWorkload, seed: int, peer: int) -> np.ndarray:
    """int32 [T][K] expert ids of rank `peer`'s tokens, in the order the gate
    emits them (descending score / draw order); never sorted by id."""
    T, E, K = w.n_tokens, w.n_experts, w.top_k
    k = _key(seed, w.wid, 0x70B, peer)
    ctr = np.arange(T * E, dtype=_U64)
    if w.routing == "uniform":
        # top-K of iid uniform keys = K experts uniformly without replacement
        score = _uniform(k, ctr).reshape(T, E)
        ids = _top_desc(score, K)
    elif w.routing == "dsv3":
        logits = _normal(k, T * E).reshape(T, E)
        z = logits - logits.max(axis=1, keepdims=True)
        p = np.exp(z)
        p /= p.sum(axis=1, keepdims=True)               # softmax scores
        per_node = E // w.n_nodes
        pn = p.reshape(T, w.n_nodes, per_node)
        top2 = -np.partition(-pn, 1, axis=2)[:, :, :2]
        node_score = top2.sum(axis=2)                   # two best experts of the node
        keep = _top_desc(node_score, w.max_nodes)       # [T][max_nodes]
        allowed = np.zeros((T, w.n_nodes), dtype=bool)
        np.put_along_axis(allowed, keep, True, axis=1)
        masked = np.where(np.repeat(allowed, per_node, axis=1), p, -1.0)
        ids = _top_desc(masked, K)
    elif w.routing == "zipf":
        order = zipf_order(w, seed)
        logw = np.empty(E, dtype=np.float64)
        logw[order] = -w.zipf_s * np.log(np.arange(1, E + 1, dtype=np.float64))
        gumbel = -np.log(-np.log(_uniform(k, ctr))).reshape(T, E)
        ids = _top_desc(logw[None, :] + gumbel, K)      # Plackett-Luce draw order
    else:
        raise ValueError(w.routing)
    return np.ascontiguousarray(ids, dtype=np.int32)


def tokens_for_rank(w: DispatchWorkload, topk: np.ndarray, rank: int) -> np.ndarray:
    """Token indices whose expert list names an expert placed on `rank`
    (ascending).  Used only to decide which payload rows are worth drawing
    when a peer's full payload would be wasteful to generate."""
    e2r = expert_to_rank(w)
    valid = (topk >= 0) & (topk < w.n_experts)
    r = np.where(valid, e2r[np.clip(topk, 0, w.n_experts - 1)], -1)
    return np.nonzero((r == rank).any(axis=1))[0].astype(np.int64)


# --------------------------------------------------------------------------
# payload draws
# --------------------------------------------------------------------------
def _row_normals(w_id: int, seed: int, peer: int, tokens: np.ndarray, hidden: int) -> np.ndarray:
    """float32 [n][hidden]; row i depends only on (seed, workload, peer, tokens[i])."""
    tokens = np.asarray(tokens, dtype=np.int64)
    base = _key(seed, w_id, 0xDA7A, peer)
    row_key = _mix(tokens.astype(_U64) ^ base)           # one stream per row
    m = (hidden + 1) // 2
    out = np.empty((len(tokens), 2 * m), dtype=np.float32)
    i2 = np.arange(m, dtype=_U64) * _U64(2)
    scale = 1.0 / 9007199254740992.0
    step = max(1, (1 << 20) // max(m, 1))               # bound the temporaries
    for lo in range(0, len(tokens), step):
        k = row_key[lo:lo + step, None]
        u1 = ((_mix(_mix(i2[None, :] ^ k) + k) >> _U64(11)).astype(np.float64) + 0.5) * scale
        u2 = ((_mix(_mix((i2 + _U64(1))[None, :] ^ k) + k) >> _U64(11)).astype(np.float64) + 0.5) * scale
        r = np.sqrt(-2.0 * np.log(u1))
        ang = (2.0 * np.pi) * u2
        out[lo:lo + step, 0::2] = r * np.cos(ang)
        out[lo:lo + step, 1::2] = r * np.sin(ang)
    return np.ascontiguousarray(out[:, :hidden])


def payload_rows(w: DispatchWorkload, seed: int, peer: int,
                 tokens: Optional[np.ndarray] = None) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Payload of the listed tokens of rank `peer` (all tokens if None).

    bf16: (uint16 [n][H] bit patterns of N(0,1) values, None).
    fp8 : (uint8 [n][H] OCP e4m3 codes, float32 [n][H/128] scales) where each
          128-element block is scaled by amax/448 and rounded to nearest even.
    """
    if tokens is None:
        tokens = np.arange(w.n_tokens, dtype=np.int64)
    x = _row_normals(w.wid, seed, peer, tokens, w.hidden)
    if w.row_format == "bf16":
        return f32_to_bf16_bits(x), None
    import torch  # CPU cast only
    n = len(tokens)
    xb = x.reshape(n, w.hidden // 128, 128)
    amax = np.abs(xb).max(axis=2)
    scale = (np.maximum(amax, 1e-12) / 448.0).astype(np.float32)
    q = np.clip(xb / scale[:, :, None], -448.0, 448.0).astype(np.float32)
    codes = torch.from_numpy(q.reshape(n, w.hidden)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    return np.ascontiguousarray(codes), np.ascontiguousarray(scale)


def payload_full(w: DispatchWorkload, seed: int, peer: int,
                 tokens: Optional[np.ndarray] = None):
    """[T][H] payload (and [T][H/128] scales for fp8) of rank `peer` in which
    only the listed tokens are drawn; the others stay zero (their pages are
    never touched).  tokens=None draws every row."""
    rows, sc = payload_rows(w, seed, peer, tokens)
    if tokens is None:
        return rows, sc
    x = np.zeros((w.n_tokens, w.hidden), dtype=rows.dtype)
    x[tokens] = rows
    s = None
    if sc is not None:
        s = np.zeros((w.n_tokens, w.hidden // 128), dtype=np.float32)
        s[tokens] = sc
    return x, s


_POOLS: Dict[tuple, np.ndarray] = {}


def payload_rows_pooled(w: DispatchWorkload, seed: int, peer: int,
                        tokens: Optional[np.ndarray] = None, pool_rows: int = 2048) -> np.ndarray:
    """bf16 payload for cases with so many rows that drawing each of them would take minutes
    (a hundred thousand rows of 7168 values): row (peer, t) is row hash(peer, t) % pool_rows of
    a pool of N(0,1) rows drawn once per (seed, workload), with its first four bf16 elements
    replaced by the row's own 64-bit hash, so that no two rows of a run are equal and a row that
    ends up in the wrong place shows.  uint16 [n][H] bit patterns.  bf16 workloads only."""
    assert w.row_format == "bf16" and w.hidden >= 4
    if tokens is None:
        tokens = np.arange(w.n_tokens, dtype=np.int64)
    tokens = np.asarray(tokens, dtype=np.int64)
    key = (seed, w.wid, w.hidden, pool_rows)
    if key not in _POOLS:
        _POOLS.clear()                                  # one pool at a time: they are large
        _POOLS[key] = f32_to_bf16_bits(_row_normals(w.wid, seed, 0x7FFFFFFF, np.arange(pool_rows), w.hidden))
    pool = _POOLS[key]
    h = _bits(_key(seed, w.wid, 0xB001, peer), tokens)
    rows = pool[(h % _U64(pool_rows)).astype(np.int64)]        # (fancy indexing copies)
    rows[:, :4] = h[:, None].view(np.uint16).reshape(len(tokens), 4)
    return rows


def allgather_shard(w: AllGatherWorkload, seed: int, rank: int) -> np.ndarray:
    """uint16 [shard_elems]: bf16 bit patterns of N(0,1) values of `rank`."""
    k = _key(seed, w.wid, 0xA6, rank)
    return f32_to_bf16_bits(_normal(k, w.shard_elems).astype(np.float32))


def topk_ids_many(w: DispatchWorkload, seed: int, peers, threads: int = 8):
    """topk_ids for several peers (numpy releases the GIL in the heavy parts)."""
    from concurrent.futures import ThreadPoolExecutor
    peers = list(peers)
    with ThreadPoolExecutor(max(1, threads)) as ex:
        return list(ex.map(lambda p: topk_ids(w, seed, p), peers))
