"""Pure-Python brute-force definitions used to pin the CPU oracle on tiny
inputs.  Written separately from oracle/ (Python ints for bitmaps, sets and
sorted() for everything else); deliberately quadratic."""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def dest_set(ids: Sequence[int], e2r: Sequence[int]) -> set:
    return {int(e2r[e]) for e in ids if e != -1}


def mask_int(ids: Sequence[int], e2r: Sequence[int]) -> int:
    m = 0
    for r in dest_set(ids, e2r):
        m |= 1 << r          # bit r <-> rank r, ranks numbered from zero
    return m


def words_to_int(words: np.ndarray) -> int:
    return sum(int(words[w]) << (64 * w) for w in range(4))


def plan_brute(topk: np.ndarray, e2r: Sequence[int]):
    """perm by O(T^2) predecessor counting; groups as runs of equal bitmaps."""
    T = topk.shape[0]
    masks = [mask_int(topk[t], e2r) for t in range(T)]
    kept = [t for t in range(T) if masks[t] != 0]
    perm = [None] * len(kept)
    for t in kept:
        before = sum(1 for u in kept if (masks[u], u) < (masks[t], t))
        perm[before] = t
    groups = []        # (mask, row_offset, row_count, n_dest)
    for i, t in enumerate(perm):
        if i == 0 or masks[t] != masks[perm[i - 1]]:
            groups.append([masks[t], i, 0, bin(masks[t]).count("1")])
        groups[-1][2] += 1
    return masks, perm, [tuple(g) for g in groups]


def dispatch_plain_brute(peers: Sequence[Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]],
                         e2r: Sequence[int], my_rank: int):
    """What unicast dispatch delivers to `my_rank`: per local expert (ascending
    id), per peer (ascending), per token (ascending) whose top-k set holds it."""
    entries: List[Tuple[int, int]] = []
    offsets = []
    for e in range(len(e2r)):
        if e2r[e] != my_rank:
            continue
        offsets.append(len(entries))
        for p, (tk, _, _) in enumerate(peers):
            for t in range(tk.shape[0]):
                if e in set(int(v) for v in tk[t]):
                    entries.append((p, t))
    offsets.append(len(entries))
    rows = [peers[p][1][t].tobytes() for p, t in entries]
    scales = [peers[p][2][t].tobytes() for p, t in entries] if peers and peers[0][2] is not None else None
    return entries, offsets, rows, scales
