"""The oracle against itself and against brute force on randomly drawn small configurations
(non-uniform expert placement, ranks without experts, padding, duplicates): the plain
definition (tier 1), the method's steps (tier 2), the packet path and the Python brute force
must all give the same delivery; plan invariants hold.  CPU only."""
import numpy as np
import pytest

from oracle import ref

import brute


def draw(rng):
    R = int(rng.choice([1, 2, 3, 5, 8, 13, 64, 65, 130, 256]))
    E = int(rng.integers(1, 3 * R + 2))
    K = int(rng.choice([1, 2, 3, 5, 8, 9]))
    T = int(rng.integers(0, 40))
    hidden = int(rng.choice([8, 16, 40]))
    e2r = rng.integers(0, R, size=E).astype(np.int32)
    return R, E, K, T, hidden, e2r


@pytest.mark.parametrize("case", range(40))
def test_all_derivations_agree(case):
    rng = np.random.default_rng(500 + case)
    R, E, K, T, hidden, e2r = draw(rng)
    counts = np.bincount(e2r, minlength=R)
    my_rank = int(np.argmax(counts)) if case % 3 else int(rng.integers(0, R))
    n_peers = int(rng.integers(1, min(R, 4) + 1))
    rb = 2 * hidden
    toks, bufs, regions = [], [], []
    for p in range(n_peers):
        tk = rng.integers(0, E, size=(T, K)).astype(np.int32)
        tk[rng.random((T, K)) < 0.25] = -1
        x = rng.integers(0, 1 << 16, size=(T, hidden), dtype=np.uint16)
        toks.append((tk, x, None))
        mask, perm, desc, st = ref.plan(tk, e2r, R, rb)
        # plan against the brute force
        bm, bperm, bgroups = brute.plan_brute(tk, e2r)
        assert [brute.words_to_int(m) for m in mask] == bm
        assert perm.tolist() == bperm
        assert [(brute.words_to_int(d["mask"]), int(d["row_offset"]), int(d["row_count"]), int(d["n_dest"]))
                for d in desc] == bgroups
        # accounting: one copy per kept token against one per (token, destination)
        dests = [len(brute.dest_set(tk[t], e2r)) for t in range(T)]
        assert int(st["multicast_bytes"]) == rb * sum(1 for d in dests if d)
        assert int(st["unicast_bytes"]) == rb * sum(dests)
        assert st["rows_per_dest"][:R].tolist() == [sum(1 for t in range(T) if r in brute.dest_set(tk[t], e2r))
                                                    for r in range(R)]
        packed, src, rtk = ref.pack(x, None, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
        regions.append(ref.deliver_packets(ref.pack_packets(x, None, tk, mask, perm), my_rank))
    cap = 10 ** 4
    plain = ref.dispatch_plain(toks, e2r, my_rank, cap)
    steps = ref.unpack(bufs, K, e2r, my_rank, rb, 0, cap)
    pkts = ref.unpack_packets(regions, K, e2r, my_rank, rb, 0, cap)
    for a, b, c in zip(plain, steps[:5], pkts[:5]):
        assert (a is None and b is None and c is None) or a.tobytes() == b.tobytes() == c.tobytes()
    entries, offsets, rows, _ = brute.dispatch_plain_brute(toks, e2r, my_rank)
    assert list(zip(plain[2].tolist(), plain[3].tolist())) == entries and plain[4].tolist() == offsets
    assert [r.tobytes() for r in plain[0]] == rows
    assert steps[5] == pkts[5] == len({(p, t) for p, t in entries})
