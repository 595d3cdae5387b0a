"""Pins of the oracle's relay step without the metadata update and of the end node's
de-duplication (ref_relay_child_unmodified, ref_unpack_dedup), against what Section 4.1's last
paragraph of "Replication and forwarding" and plain set arithmetic fix.  CPU only."""
import numpy as np
import pytest

from oracle import ref
from paper_2605_22428_amd import workloads as W

import brute


def _send(w, seed, p):
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, seed, p)
    x, sc = W.payload_rows(w, seed, p)
    _, perm, desc, st = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    packed, src, rtk = ref.pack(x, sc, tk, perm)
    return tk, x, sc, (desc, packed, src, rtk)


def _ranks_of(words):
    m = brute.words_to_int(words)
    return {r for r in range(256) if (m >> r) & 1}


def concat(bufs):
    """Several received buffers of one source as one region: descriptors one after the other, row
    ranges rebased (what lands in a peer's receive region over more than one path)."""
    descs, rows, src, rtk, off = [], [], [], [], 0
    for d, r, s, t in bufs:
        d = d.copy()
        d["row_offset"] += np.uint32(off)
        off += len(r)
        descs.append(d); rows.append(r); src.append(s); rtk.append(t)
    return (np.concatenate(descs), np.concatenate(rows), np.concatenate(src), np.concatenate(rtk))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_unmodified_child_is_the_updated_child_with_the_parents_bitmap(seed):
    """The copies a relay makes do not depend on whether it rewrites the metadata: same groups,
    rows, row metadata and row ranges per hop; only the bitmap (and its popcount) is the parent's."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("t", 33, 12, 24, 3, 60, 64, "bf16", "uniform")
    _, _, _, (desc, rows, src, rtk) = _send(w, seed, 1)
    n_hops = 4
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    for h in range(n_hops):
        upd = ref.relay_child(desc, rows, src, rtk, next_hop, n_hops, h)
        raw = ref.relay_child(desc, rows, src, rtk, next_hop, n_hops, h, update_metadata=False)
        for a, b in zip(upd[1:], raw[1:]):
            assert a.tobytes() == b.tobytes()
        assert upd[0]["row_offset"].tolist() == raw[0]["row_offset"].tolist()
        assert upd[0]["row_count"].tolist() == raw[0]["row_count"].tolist()
        kept = [g for g in range(len(desc)) if any(next_hop[r] == h for r in _ranks_of(desc["mask"][g]))]
        assert len(raw[0]) == len(kept)
        for cg, g in enumerate(kept):
            assert raw[0]["mask"][cg].tolist() == desc["mask"][g].tolist()
            assert int(raw[0]["n_dest"][cg]) == len(_ranks_of(desc["mask"][g])) == int(desc["n_dest"][g])
            assert _ranks_of(upd[0]["mask"][cg]) <= _ranks_of(raw[0]["mask"][cg])
            assert int(raw[0]["reserved0"][cg]) == 0
    # a table with a single hop forwards the parent as it is, either way
    one = np.zeros(w.n_ranks, dtype=np.int32)
    for flag in (True, False):
        c = ref.relay_child(desc, rows, src, rtk, one, 1, 0, update_metadata=flag)
        assert c[0].tobytes() == desc.tobytes() and c[1].tobytes() == rows.tobytes()


def test_dedup_takes_the_first_row_of_every_token_hand_worked():
    """One peer, five rows with source tokens 3, 5, 3, 7, 5, all for the one local expert: rows 0,
    1 and 3 are taken (tokens 3, 5, 7), two repeats are dropped, and the output is in token order."""
    e2r = np.array([0, 1], dtype=np.int32)
    desc = np.zeros(1, dtype=ref.DESC)
    desc["mask"][0, 0] = 0b11
    desc["row_count"][0] = 5
    desc["n_dest"][0] = 2
    rows = (np.arange(5, dtype=np.uint8)[:, None] + np.zeros((5, 16), dtype=np.uint8))     # row i is filled with i
    src = np.array([3, 5, 3, 7, 5], dtype=np.int32)
    rtk = np.array([[1]] * 5, dtype=np.int32)
    out, _, sp, st, offs, (taken, dropped) = ref.unpack_dedup([(desc, rows, src, rtk)], 1, e2r, 1, 16, 0, 8)
    assert (taken, dropped) == (3, 2)
    assert st.tolist() == [3, 5, 7] and sp.tolist() == [0, 0, 0] and offs.tolist() == [0, 3]
    assert out[:, 0].tolist() == [0, 1, 3]
    with pytest.raises(ref.OracleError):              # the plain receive side refuses the repeats
        ref.unpack([(desc, rows, src, rtk)], 1, e2r, 1, 16, 0, 8)


@pytest.mark.parametrize("seed", [1, 2])
def test_dedup_without_repeats_is_unpack(seed):
    w = W.DispatchWorkload("t", 34, 8, 16, 2, 70, 64, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    my_rank = 5
    bufs = []
    for p in range(w.n_ranks):
        _, _, _, (desc, rows, src, rtk) = _send(w, seed, p)
        bufs.append(ref.deliver(desc, rows, src, rtk, my_rank))
    a = ref.unpack(bufs, w.top_k, e2r, my_rank, w.row_bytes, 0, 400)
    b = ref.unpack_dedup(bufs, w.top_k, e2r, my_rank, w.row_bytes, 0, 400)
    for x, y in zip(a[:5], b[:5]):
        assert (x is None and y is None) or x.tobytes() == y.tobytes()
    assert b[5] == (a[5], 0)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_delivery_through_relays_that_do_not_update_equals_direct_delivery(seed):
    """A loop-free deployment of the option: every source has a direct link to some ranks and
    reaches the others through relay ranks; relays forward once (to the ranks they have a direct
    link to, whatever the source already served) and end nodes never forward.  With unmodified
    bitmaps a destination then holds the same (source, token) row once per path; with the end
    node's de-duplication what it delivers is exactly what direct delivery gives (the plain
    definition), and without it the repeats are an input error."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("t", 35, 10, 20, 3, 40, 32, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    R = w.n_ranks
    relays = [2, 7]
    toks = []
    regions = {d: [] for d in range(R)}            # per destination: one region per source
    n_dup_total = 0
    for s in range(R):
        tk, x, sc, parent = _send(w, seed, s)
        toks.append((tk, x, sc))
        # the source's table: hop 0 = direct link (ranks it reaches itself), hop 1 + j = through relay j
        via = rng.integers(0, 1 + len(relays), size=R).astype(np.int32)
        via[s] = 0
        for j, rl in enumerate(relays):
            via[rl] = 0 if rl == s else via[rl]
        arrivals = {d: [] for d in range(R)}
        direct = ref.relay_child(*parent, via, 1 + len(relays), 0, update_metadata=False)
        for d in range(R):
            if via[d] == 0:
                arrivals[d].append(ref.deliver(*direct, d))
        for j, rl in enumerate(relays):
            to_relay = ref.relay_child(*parent, via, 1 + len(relays), 1 + j, update_metadata=False)
            if len(to_relay[0]) == 0:
                continue
            # the relay forwards to every rank named in the (unmodified) bitmaps that it links to directly:
            # here all ranks but the source; identity table = one hop per rank
            ident = np.arange(R, dtype=np.int32)
            for d in range(R):
                if d == s or d == rl:
                    continue
                child = ref.relay_child(*to_relay, ident, R, d, update_metadata=False)
                arrivals[d].append(ref.deliver(*child, d))
            # (the relay itself is an end node for its own rows only if the source sent them its way)
            if via[rl] == 1 + j:
                arrivals[rl].append(ref.deliver(*to_relay, rl))
        for d in range(R):
            got = [a for a in arrivals[d] if len(a[1])]
            if got:
                regions[d].append(concat(got))
            else:
                regions[d].append((np.zeros(0, dtype=ref.DESC), np.zeros((0, w.row_bytes), np.uint8),
                                   np.zeros(0, np.int32), np.zeros((0, w.top_k), np.int32)))
    for d in (0, 2, 5, 9):
        cap = 4 * sum(len(r[1]) for r in regions[d]) + 4
        want = ref.dispatch_plain(toks, e2r, d, cap)
        got = ref.unpack_dedup(regions[d], w.top_k, e2r, d, w.row_bytes, 0, cap)
        for name, a, b in zip(("rows", "scales", "src_peer", "src_token", "offsets"), got[:5], want[:5]):
            assert (a is None and b is None) or a.tobytes() == b.tobytes(), (d, name)
        taken, dropped = got[5]
        assert taken + dropped == sum(len(r[1]) for r in regions[d])
        n_dup_total += dropped
        if dropped:
            with pytest.raises(ref.OracleError):
                ref.unpack(regions[d], w.top_k, e2r, d, w.row_bytes, 0, cap)
    assert n_dup_total > 0          # (the construction does produce repeats)


@pytest.mark.parametrize("seed", [1, 2])
def test_unmodified_packets_child_is_the_kept_parent_packets_verbatim(seed):
    """Packets form of the option: per hop the same packets are kept as by the updating relay (a
    packet travels to a hop iff its bitmap names a rank behind it, brute force over bits), each one
    byte for byte the parent's; the updated child differs from it in the bitmap bytes only."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("t", 36, 12, 24, 3, 50, 64, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, seed, 0)
    x, sc = W.payload_rows(w, seed, 0)
    mask, perm, _, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    pk = ref.pack_packets(x, sc, tk, mask, perm)
    n_hops = 5
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    total = 0
    for h in range(n_hops):
        raw = ref.relay_packets_child(pk, next_hop, n_hops, h, update_metadata=False)
        upd, _, _ = ref.relay_packets_child(pk, next_hop, n_hops, h)
        keep = [i for i in range(len(pk))
                if any(next_hop[r] == h for r in range(w.n_ranks)
                       if (int.from_bytes(pk[i, :32].tobytes(), "little") >> r) & 1)]
        assert raw.tobytes() == pk[keep].tobytes()
        assert upd[:, 32:].tobytes() == raw[:, 32:].tobytes()
        total += len(raw)
    assert total > len(pk)           # (some packet does travel over more than one hop)
    with pytest.raises(ref.OracleError):
        ref.relay_packets_child(pk, np.zeros(2, np.int32), 1, 0, update_metadata=False)    # bitmaps name ranks >= 2
