"""Pins of the oracle's packet functions (bitmap and row metadata embedded in front of every
row, Section 6.4) against a hand-written header, a parser written separately in Python, the
plain definition of a dispatch, and the descriptor-table path.  CPU only."""
import json
import os
import struct

import numpy as np
import pytest

from oracle import ref
from paper_2605_22428_amd import workloads as W

import brute


def _sender(w, seed, p, edit=None):
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, seed, p)
    if edit is not None:
        edit(tk)
    x, sc = W.payload_rows(w, seed, p)
    mask, perm, desc, st = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    return tk, x, sc, mask, perm, desc


def _parse(header: bytes):
    """Independent parser: struct.unpack on the documented offsets."""
    words = struct.unpack_from("<4Q", header, 0)
    token, k = struct.unpack_from("<iI", header, 32)
    ids = struct.unpack_from("<%di" % k, header, 40)
    return sum(w << (64 * i) for i, w in enumerate(words)), token, k, list(ids)


def test_hand_written_header(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "packet_header_example.json")))
    K = g["top_k"]
    e2r = np.array(g["expert_to_rank"], dtype=np.int32)
    T = 259
    tk = np.full((T, K), -1, dtype=np.int32)
    tk[g["token_index"]] = g["expert_ids"]
    tk[g["second_token"]["token_index"]] = g["second_token"]["expert_ids"]
    x = (np.arange(T * 8, dtype=np.uint16) * 3 + 1).reshape(T, 8)
    mask, perm, desc, st = ref.plan(tk, e2r, g["n_ranks"], 16)
    pk = ref.pack_packets(x, None, tk, mask, perm)
    assert ref.packet_header_bytes(K) == g["header_bytes"] and pk.shape == (2, g["header_bytes"] + 16)
    by_token = {int(t): pk[i] for i, t in enumerate(perm)}
    for tok, key in ((g["token_index"], "header_hex_token_5"),
                     (g["second_token"]["token_index"], "header_hex_token_258")):
        want = bytes.fromhex(g[key].replace(" ", ""))
        want = want + bytes(g["header_bytes"] - len(want))
        assert by_token[tok][: g["header_bytes"]].tobytes() == want
        assert by_token[tok][g["header_bytes"]:].tobytes() == x[tok].tobytes()
    # the bitmap in the hand-written header is the one the stated destinations give
    m, _, _, _ = _parse(bytes.fromhex(g["header_hex_token_258"].replace(" ", "")))
    assert m == sum(1 << r for r in g["second_token"]["destination_ranks"])


def test_header_size_and_the_papers_overhead_example(golden_dir):
    a = json.load(open(os.path.join(golden_dir, "paper_arithmetic.json")))["in_payload_bitmap_overhead"]
    # Section 6.4: 1024 bit in front of 4096 byte = 3.13 %; the header here is those 128 bytes
    assert a["bitmap_bits"] // 8 == ref.packet_header_bytes(8) == 128
    assert abs(100.0 * ref.packet_header_bytes(8) / a["payload_bytes"] - a["printed_percent"]) <= 0.005
    for K in range(0, 65):
        hb = ref.packet_header_bytes(K)
        assert hb % 128 == 0 and hb >= 40 + 4 * K and hb - 128 < 40 + 4 * K
    assert ref.packet_header_bytes(22) == 128 and ref.packet_header_bytes(23) == 256


@pytest.mark.parametrize("fmt,seed", [("bf16", 1), ("fp8", 2)])
def test_fields_against_a_separate_parser(fmt, seed):
    w = W.DispatchWorkload("t", 31, 70, 140, 5, 60, 512, fmt, "uniform")
    e2r = W.expert_to_rank(w)

    def edit(tk):
        tk[::4, 2] = -1
        tk[1::6, 1] = tk[1::6, 0]
        tk[9] = -1
    tk, x, sc, mask, perm, desc = _sender(w, seed, 3, edit)
    pk = ref.pack_packets(x, sc, tk, mask, perm)
    packed, src, rtk = ref.pack(x, sc, tk, perm)
    hb = ref.packet_header_bytes(w.top_k)
    assert pk.shape == (len(perm), hb + w.row_bytes) and 9 not in perm.tolist()
    for i in range(len(perm)):
        m, token, k, ids = _parse(pk[i, :hb].tobytes())
        assert (token, k, ids) == (int(perm[i]), w.top_k, tk[perm[i]].tolist())
        assert m == brute.mask_int(tk[perm[i]], e2r)
        assert not pk[i, 40 + 4 * k:hb].any()
        assert pk[i, hb:].tobytes() == packed[i].tobytes()


@pytest.mark.parametrize("fmt", ["bf16", "fp8"])
@pytest.mark.parametrize("seed,my_rank", [(1, 0), (2, 6), (3, 11)])
def test_delivery_equals_the_plain_definition_and_the_descriptor_path(fmt, seed, my_rank):
    w = W.DispatchWorkload("t", 32, 12, 36, 4, 40, 512, fmt, "uniform")
    e2r = W.expert_to_rank(w)
    xrb = w.hidden * (2 if fmt == "bf16" else 1)
    srb = w.row_bytes - xrb
    rng = np.random.default_rng(seed)
    toks, filtered, complete, shuffled, bufs = [], [], [], [], []
    for p in range(w.n_ranks):
        def edit(tk):
            tk[p % 5::7, 3] = -1
            tk[(p + 2) % 9::9, 1] = tk[(p + 2) % 9::9, 0]
        tk, x, sc, mask, perm, desc = _sender(w, seed, p, edit)
        pk = ref.pack_packets(x, sc, tk, mask, perm)
        toks.append((tk, x, sc))
        complete.append(pk)
        kept = ref.deliver_packets(pk, my_rank)
        filtered.append(kept)
        shuffled.append(kept[rng.permutation(len(kept))])
        packed, src, rtk = ref.pack(x, sc, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
        # the simulated network keeps exactly the packets of tokens with an expert on my_rank
        want = [t for t in perm if my_rank in brute.dest_set(tk[t], e2r)]
        assert [struct.unpack_from("<i", k.tobytes(), 32)[0] for k in kept] == want
    cap = 10 ** 4
    plain = ref.dispatch_plain(toks, e2r, my_rank, cap)
    table = ref.unpack(bufs, w.top_k, e2r, my_rank, xrb, srb, cap)
    for name, peers in (("filtered", filtered), ("complete buffers", complete), ("any arrival order", shuffled)):
        got = ref.unpack_packets(peers, w.top_k, e2r, my_rank, xrb, srb, cap)
        for a, b in zip(got[:5], plain):
            assert (a is None and b is None) or a.tobytes() == b.tobytes(), name
        assert got[5] == table[5] == sum(len(f) for f in filtered), name
        for a, b in zip(got[:5], table[:5]):
            assert (a is None and b is None) or a.tobytes() == b.tobytes(), name
    # brute force in Python, for the record order
    entries, offsets, rows, _ = brute.dispatch_plain_brute(toks, e2r, my_rank)
    got = ref.unpack_packets(filtered, w.top_k, e2r, my_rank, xrb, srb, cap)
    assert list(zip(got[2].tolist(), got[3].tolist())) == entries and got[4].tolist() == offsets


def test_inconsistent_packets_are_refused():
    w = W.DispatchWorkload("t", 33, 4, 8, 2, 12, 64, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tk, x, sc, mask, perm, desc = _sender(w, 1, 0)
    pk = ref.deliver_packets(ref.pack_packets(x, sc, tk, mask, perm), 1)
    assert len(pk) >= 2
    ok = ref.unpack_packets([pk], 2, e2r, 1, 128, 0, 100)
    assert ok[5] == len(pk)
    bad = pk.copy(); bad[0, 36] = 3                       # K in the header differs from the configuration
    with pytest.raises(ref.OracleError):
        ref.unpack_packets([bad], 2, e2r, 1, 128, 0, 100)
    dup = np.concatenate([pk, pk[:1]])                    # the same token twice from one peer
    with pytest.raises(ref.OracleError):
        ref.unpack_packets([dup], 2, e2r, 1, 128, 0, 100)
    with pytest.raises(ref.OracleError):
        ref.unpack_packets([pk], 2, e2r, 1, 128, 0, 0)    # no room


# ------------------------------------------------------------------ relay of packets
def _ranks(header: bytes):
    m, _, _, _ = _parse(header)
    return {r for r in range(256) if (m >> r) & 1}


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_relayed_copies_partition_every_bitmap_and_match_the_descriptor_path(seed):
    """Section 4.1, update of in-packet metadata: the copies of one packet name disjoint sets
    that together are the parent's; the number of copies is the number of distinct next hops."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("t", 34, 12, 24, 3, 50, 64, "bf16", "uniform")
    tk, x, sc, mask, perm, desc = _sender(w, seed, 0)
    pk = ref.pack_packets(x, sc, tk, mask, perm)
    packed, src, rtk = ref.pack(x, sc, tk, perm)
    n_hops = 5
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    seen = [set() for _ in range(len(pk))]
    copies_total = 0
    for h in range(n_hops):
        child, copies, dests = ref.relay_packets_child(pk, next_hop, n_hops, h)
        keep = [i for i in range(len(pk)) if any(next_hop[r] == h for r in _ranks(pk[i, :128].tobytes()))]
        assert len(child) == len(keep)
        copies_total += len(child)
        for c, i in zip(child, keep):
            sub = _ranks(c[:128].tobytes())
            assert sub == {r for r in _ranks(pk[i, :128].tobytes()) if next_hop[r] == h}
            assert not (sub & seen[i])
            seen[i] |= sub
            assert c[32:].tobytes() == pk[i, 32:].tobytes()        # everything but the bitmap is unchanged
        # the descriptor-table relay keeps the same rows with the same restricted bitmaps
        d2, r2, s2, t2 = ref.relay_child(desc, packed, src, rtk, next_hop, n_hops, h)
        rows_desc = [(brute.words_to_int(d2["mask"][g]), int(s2[int(d2["row_offset"][g]) + k]))
                     for g in range(len(d2)) for k in range(int(d2["row_count"][g]))]
        rows_pk = [(_parse(c[:128].tobytes())[0], _parse(c[:128].tobytes())[1]) for c in child]
        assert rows_pk == rows_desc
        assert child[:, 128:].tobytes() == r2.tobytes()
    assert all(seen[i] == _ranks(pk[i, :128].tobytes()) for i in range(len(pk)))
    assert copies == copies_total == sum(len({int(next_hop[r]) for r in _ranks(p[:128].tobytes())}) for p in pk)
    assert dests == sum(len(_ranks(p[:128].tobytes())) for p in pk)


def test_delivery_through_two_levels_of_relays_equals_direct_delivery():
    """Section 4.3.3: the recursion ends in plain writes and delivers what a direct MultiWrite
    delivers.  Two servers of four devices: first hop per server, second hop per device."""
    w = W.DispatchWorkload("t", 35, 8, 24, 4, 40, 128, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    my_rank = 6
    toks, direct, relayed = [], [], []
    for p in range(w.n_ranks):
        tk, x, sc, mask, perm, desc = _sender(w, 4, p)
        toks.append((tk, x, sc))
        pk = ref.pack_packets(x, sc, tk, mask, perm)
        direct.append(ref.deliver_packets(pk, my_rank))
        to_server = np.array([r // 4 for r in range(8)], dtype=np.int32)
        at_server, _, _ = ref.relay_packets_child(pk, to_server, 2, my_rank // 4)
        to_device = np.array([r % 4 for r in range(8)], dtype=np.int32)      # only this server's ranks remain
        mine, _, _ = ref.relay_packets_child(at_server, to_device, 4, my_rank % 4)
        for c in mine:
            assert _ranks(c[:128].tobytes()) == {my_rank}                    # down to a plain write
        relayed.append(mine)
    cap = 10 ** 4
    a = ref.unpack_packets(direct, w.top_k, e2r, my_rank, w.row_bytes, 0, cap)
    b = ref.unpack_packets(relayed, w.top_k, e2r, my_rank, w.row_bytes, 0, cap)
    plain = ref.dispatch_plain(toks, e2r, my_rank, cap)
    for u, v, z in zip(a[:5], b[:5], plain):
        assert (u is None and v is None) or u.tobytes() == v.tobytes() == z.tobytes()


def test_relay_tables_that_cannot_be_followed_are_refused():
    w = W.DispatchWorkload("t", 36, 4, 8, 2, 12, 64, "bf16", "uniform")
    tk, x, sc, mask, perm, desc = _sender(w, 1, 0)
    pk = ref.pack_packets(x, sc, tk, mask, perm)
    with pytest.raises(ref.OracleError):
        ref.relay_packets_child(pk, np.array([0, 1, 2, 3], np.int32), 3, 0)      # hop 3 does not exist
    with pytest.raises(ref.OracleError):
        ref.relay_packets_child(pk, np.array([0, 1], np.int32), 2, 0)            # bitmaps name ranks 2, 3
