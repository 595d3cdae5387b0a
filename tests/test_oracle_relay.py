"""Pins of the oracle's relay step (ref_relay_child, ref_relay_accounting) against what the
paper and plain set arithmetic fix.  CPU only."""
import json
import os
from math import comb

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
    return tk, x, sc, (desc, packed, src, rtk), st


def _ranks_of(words):
    m = brute.words_to_int(words)
    return {r for r in range(256) if (m >> r) & 1}


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_children_partition_every_parent_bitmap(seed):
    """Section 4.1, update of in-packet metadata: copies leaving through different hops name
    disjoint destination sets, together exactly the parent's; Section 4.3.3 rule 3."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("t", 31, 12, 24, 3, 50, 64, "bf16", "uniform")
    _, _, _, parent, _ = _send(w, seed, 0)
    desc, rows, src, rtk = parent
    n_hops = 5
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    seen = [set() for _ in range(len(desc))]
    total_rows = 0
    for h in range(n_hops):
        d2, r2, s2, t2 = ref.relay_child(desc, rows, src, rtk, next_hop, n_hops, h)
        want = [g for g in range(len(desc)) if any(next_hop[r] == h for r in _ranks_of(desc["mask"][g]))]
        assert len(d2) == len(want)
        off = 0
        for cg, g in enumerate(want):
            sub = _ranks_of(d2["mask"][cg])
            assert sub == {r for r in _ranks_of(desc["mask"][g]) if next_hop[r] == h}
            assert not (sub & seen[g])
            seen[g] |= sub
            assert int(d2["n_dest"][cg]) == len(sub) and int(d2["reserved0"][cg]) == 0
            assert int(d2["row_offset"][cg]) == off and int(d2["row_count"][cg]) == int(desc["row_count"][g])
            a = int(desc["row_offset"][g])
            n = int(desc["row_count"][g])
            assert r2[off:off + n].tobytes() == rows[a:a + n].tobytes()
            assert s2[off:off + n].tolist() == src[a:a + n].tolist()
            assert t2[off:off + n].tobytes() == rtk[a:a + n].tobytes()
            off += n
        assert off == len(r2)
        total_rows += off
    for g in range(len(desc)):
        assert seen[g] == _ranks_of(desc["mask"][g])
    fwd, uni, rph = ref.relay_accounting(desc, w.row_bytes, next_hop, n_hops)
    assert fwd == total_rows * w.row_bytes and int(rph.sum()) == total_rows
    assert uni == w.row_bytes * sum(int(desc["row_count"][g]) * len(_ranks_of(desc["mask"][g]))
                                    for g in range(len(desc)))


def test_identity_table_is_unicast_delivery():
    """One hop per rank: every child is what ref_deliver hands that rank, with a single-bit
    bitmap (Section 4.3.3 rule 2: one destination left = a standard write), and the relay
    makes exactly as many copies as unicast would."""
    w = W.DispatchWorkload("t", 32, 8, 16, 2, 64, 64, "bf16", "uniform")
    _, _, _, parent, st = _send(w, 5, 3)
    desc, rows, src, rtk = parent
    ident = np.arange(w.n_ranks, dtype=np.int32)
    for r in range(w.n_ranks):
        d2, r2, s2, t2 = ref.relay_child(desc, rows, src, rtk, ident, w.n_ranks, r)
        d1, r1, s1, t1 = ref.deliver(desc, rows, src, rtk, r)
        assert r2.tobytes() == r1.tobytes() and s2.tolist() == s1.tolist() and t2.tobytes() == t1.tobytes()
        assert d2["row_offset"].tolist() == d1["row_offset"].tolist()
        assert d2["row_count"].tolist() == d1["row_count"].tolist()
        assert all(_ranks_of(m) == {r} for m in d2["mask"]) and set(d2["n_dest"].tolist()) <= {1}
    fwd, uni, rph = ref.relay_accounting(desc, w.row_bytes, ident, w.n_ranks)
    assert fwd == uni == int(st["unicast_bytes"])
    assert rph.tolist() == st["rows_per_dest"][: w.n_ranks].tolist()


def test_single_hop_returns_the_parent():
    w = W.DispatchWorkload("t", 33, 8, 16, 2, 40, 512, "fp8", "uniform")
    _, _, _, parent, st = _send(w, 6, 1)
    desc, rows, src, rtk = parent
    one = np.zeros(w.n_ranks, dtype=np.int32)
    d2, r2, s2, t2 = ref.relay_child(desc, rows, src, rtk, one, 1, 0)
    assert d2.tobytes() == desc.tobytes() and r2.tobytes() == rows.tobytes()
    assert s2.tolist() == src.tolist() and t2.tobytes() == rtk.tobytes()
    fwd, uni, _ = ref.relay_accounting(desc, w.row_bytes, one, 1)
    assert fwd == int(st["multicast_bytes"]) and uni == int(st["unicast_bytes"])


def _two_server_tables(n_per):
    """Forwarding tables of a 2-server system (Section 3.2): direct links inside a server, one
    link to the same-index device of the other server.  Hop ids: 0..n_per-1 = local device,
    n_per = the remote server.  Returns next_hop[source rank] and n_hops."""
    R = 2 * n_per
    tables = []
    for s in range(R):
        t = np.empty(R, dtype=np.int32)
        for r in range(R):
            t[r] = (r % n_per) if r // n_per == s // n_per else n_per
        tables.append(t)
    return tables, n_per + 1


def test_delivery_through_relays_equals_direct_delivery():
    """Section 4.3.4 (drop-in replacement) with Section 3.2's topology: every rank receives,
    through the same-index relay of the other server, exactly what direct delivery gives --
    each (token, destination) once, no duplicates (Section 4.1, metadata update)."""
    n_per = 4
    w = W.DispatchWorkload("t", 34, 2 * n_per, 16, 3, 30, 64, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tables, n_hops = _two_server_tables(n_per)
    sends = [_send(w, 9, p) for p in range(w.n_ranks)]
    toks = [(s[0], s[1], s[2]) for s in sends]
    for d in (0, 5):
        bufs = []
        for p in range(w.n_ranks):
            parent = sends[p][3]
            if p // n_per == d // n_per:
                buf = ref.relay_child(*parent, tables[p], n_hops, d % n_per)
            else:
                relay = (p % n_per) + (d // n_per) * n_per           # same index, destination's server
                at_relay = ref.relay_child(*parent, tables[p], n_hops, n_per)
                assert all(_ranks_of(m) <= set(range((d // n_per) * n_per, (d // n_per + 1) * n_per))
                           for m in at_relay[0]["mask"])
                buf = ref.relay_child(*at_relay, tables[relay], n_hops, d % n_per)
            assert all(_ranks_of(m) == {d} for m in buf[0]["mask"])
            direct = ref.deliver(*parent, d)
            assert buf[1].tobytes() == direct[1].tobytes() and buf[2].tolist() == direct[2].tolist()
            bufs.append(buf)
        cap = w.n_ranks * w.n_tokens * 2
        o_relayed = ref.unpack(bufs, w.top_k, e2r, d, 2 * w.hidden, 0, cap)
        o_plain = ref.dispatch_plain(toks, e2r, d, cap)
        for a, b in zip(o_relayed[:5], o_plain[:5]):
            if a is not None:
                assert np.asarray(a).tobytes() == np.asarray(b).tobytes()


def test_paper_cross_server_example(golden_dir):
    ex = json.load(open(os.path.join(golden_dir, "paper_relay_example.json")))
    n_per = ex["npus_per_server"]
    R = ex["servers"] * n_per
    dests = ex["destinations_server0"] + ex["destinations_server1"]
    # one token, one expert per rank: its top-8 are the eight destination ranks
    topk = np.array([dests], dtype=np.int32)
    e2r = np.arange(R, dtype=np.int32)
    x = np.arange(32, dtype=np.uint8).reshape(1, 32)
    _, perm, desc, st = ref.plan(topk, e2r, R, 32)
    packed, src, rtk = ref.pack(x, None, topk, perm)
    tables, n_hops = _two_server_tables(n_per)
    s = ex["source_rank"]
    fwd, uni, rph = ref.relay_accounting(desc, 32, tables[s], n_hops)
    assert uni // 32 == ex["unicast_copies_from_source"]
    assert fwd // 32 == ex["multicast_copies_from_source"]
    assert int(rph[n_per]) == ex["cross_server_copies_multicast"]
    assert len(ex["destinations_server1"]) == ex["cross_server_copies_unicast"]
    at_relay = ref.relay_child(desc, packed, src, rtk, tables[s], n_hops, n_per)
    assert _ranks_of(at_relay[0]["mask"][0]) == set(ex["destinations_server1"])
    fwd2, uni2, rph2 = ref.relay_accounting(at_relay[0], 32, tables[ex["relay_rank"]], n_hops)
    assert fwd2 // 32 == uni2 // 32 == ex["copies_made_by_relay"] and int(rph2[n_per]) == 0
    for r in ex["destinations_server1"]:
        leaf = ref.relay_child(*at_relay, tables[ex["relay_rank"]], n_hops, r % n_per)
        assert _ranks_of(leaf[0]["mask"][0]) == {r} and leaf[1].tobytes() == x.tobytes()


def test_cross_server_copy_count_closed_form():
    """2 x 8 devices, 64 experts, top-8 uniform (Section 6.1's dispatch workload): a token
    needs a cross-server copy with probability 1 - C(32,8)/C(64,8); unicast sends it to
    8 (1 - C(60,8)/C(64,8)) remote devices on average."""
    n_per, E, K, T = 8, 64, 8, 6000
    w = W.DispatchWorkload("t", 35, 2 * n_per, E, K, T, 16, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, 11, 0)
    _, perm, desc, st = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    tables, n_hops = _two_server_tables(n_per)
    fwd, uni, rph = ref.relay_accounting(desc, w.row_bytes, tables[0], n_hops)
    p_cross = 1.0 - comb(32, 8) / comb(64, 8)
    mean_remote = 8.0 * (1.0 - comb(60, 8) / comb(64, 8))
    assert abs(rph[n_per] / T - p_cross) < 4 * np.sqrt(p_cross * (1 - p_cross) / T) + 1e-9
    remote_unicast = int(st["rows_per_dest"][n_per:2 * n_per].sum())
    assert abs(remote_unicast / T - mean_remote) < 0.06          # sd of the mean ~ 0.017
    assert uni == int(st["unicast_bytes"])


def test_relay_rejects_bad_tables_and_bitmaps():
    w = W.DispatchWorkload("t", 36, 8, 16, 2, 10, 16, "bf16", "uniform")
    _, _, _, parent, _ = _send(w, 1, 0)
    bad = np.zeros(w.n_ranks, dtype=np.int32)
    bad[3] = 7
    with pytest.raises(ref.OracleError):
        ref.relay_child(*parent, bad, 2, 0)
    with pytest.raises(ref.OracleError):
        ref.relay_child(*parent, np.zeros(w.n_ranks, dtype=np.int32), 1, 1)
    short = np.zeros(4, dtype=np.int32)                              # bitmaps name ranks the table lacks
    with pytest.raises(ref.OracleError):
        ref.relay_child(*parent, short, 1, 0)


# ---------------------------------------------------------------- AllGather with a two-segment fragment
def test_allgather_split_point_reproduces_the_papers_model(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "paper_arithmetic.json")))["allgather_tp4_full_mesh"]
    s, w = 16 << 20, 1.0

    def latency(a, copies):            # the slower of the two paths, in units of s/w
        return max(a / w, (s - a) * copies / w) / (s / w)

    a_mc = ref.allgather_split_point(s, w, w, g["copies_multicast"])
    a_uc = ref.allgather_split_point(s, w, w, g["copies_unicast"])
    assert a_mc == s // 2 and a_uc == 3 * s // 4
    assert latency(a_mc, 1) == g["latency_multicast"] and latency(a_uc, 3) == g["latency_unicast_multipath"]
    assert latency(s, 1) == g["latency_direct_only"]
    assert 1 - latency(a_mc, 1) / latency(s, 1) == g["reduction_vs_baseline"]
    assert round(100 * (1 - latency(a_mc, 1) / latency(a_uc, 3))) == g["reduction_vs_unicast_multipath_printed_percent"]
    # the balanced point is the minimum of the slower path over all splits
    for copies, wd, wr in [(1, 1.0, 1.0), (3, 1.0, 1.0), (1, 56.0, 25.0), (2, 3.0, 7.0)]:
        a = ref.allgather_split_point(s, wd, wr, copies)
        t = lambda x: max(x / wd, (s - x) * copies / wr)
        assert a % 16 == 0 and 0 <= a <= s
        assert all(t(a) <= t(x) * (1 + 1e-6) for x in range(0, s + 1, s // 64))
    for bad in [(s + 8, 1.0, 1.0, 1), (s, 0.0, 1.0, 1), (s, 1.0, -1.0, 1), (s, 1.0, 1.0, 0)]:
        with pytest.raises(ref.OracleError):
            ref.allgather_split_point(*bad)


@pytest.mark.parametrize("direct", [0, 16, 4096, 8000, 16384])
def test_allgather_split_is_still_concatenation(direct):
    w = W.AllGatherWorkload("ags", 43, 8, 8192)          # 16 KiB fragments
    s = w.shard_bytes
    shards = [W.allgather_shard(w, 5, r).view(np.uint8) for r in range(w.n_ranks)]
    d, st = ref.plan_allgather_split(w.n_ranks, s, direct)
    full = brute.words_to_int(d[0]["mask"])
    assert full == (1 << w.n_ranks) - 1 == brute.words_to_int(d[1]["mask"])
    assert (int(d[0]["row_offset"]), int(d[0]["row_count"])) == (0, direct // 16)
    assert (int(d[1]["row_offset"]), int(d[1]["row_count"])) == (direct // 16, (s - direct) // 16)
    assert int(st["n_groups"]) == 2 and int(st["n_rows"]) == s // 16
    assert int(st["multicast_bytes"]) == direct * w.n_ranks + (s - direct)
    assert int(st["unicast_bytes"]) == s * w.n_ranks
    # the two pieces travel separately (and land in separate regions)
    dpieces = [np.ascontiguousarray(x[:direct]) for x in shards]
    rpieces = [np.ascontiguousarray(x[direct:]) for x in shards]
    out = ref.unpack_allgather_split(dpieces, rpieces, s, direct)
    assert out.tobytes() == np.concatenate(shards).tobytes() == ref.unpack_allgather(shards).tobytes()
    if direct == s:                       # everything direct: the plain AllGather accounting
        _, st1 = ref.plan_allgather(w.n_ranks, s)
        assert int(st["multicast_bytes"]) == int(st1["unicast_bytes"])
    if direct == 0:                       # everything relayed once
        _, st1 = ref.plan_allgather(w.n_ranks, s)
        assert int(st["multicast_bytes"]) == int(st1["multicast_bytes"])


def test_allgather_split_rejects_bad_split_points():
    for args in [(8, 1024, 8), (8, 1024, 2048), (8, 1024, -16), (8, 1000, 0), (300, 1024, 0)]:
        with pytest.raises(ref.OracleError):
            ref.plan_allgather_split(*args)
