"""Pins for the CPU oracle: everything here runs without a GPU and checks
oracle/ against things other than itself -- brute force written separately
in Python, closed forms, library routines in special cases, invariants from
the paper's statement of MultiWrite, a hand-worked example and the paper's
printed arithmetic."""
import json
import math
import os

import numpy as np
import pytest

from oracle import ref
from paper_2605_22428_amd import workloads as W

from brute import dest_set, dispatch_plain_brute, mask_int, plan_brute, words_to_int


def _rand_topk(rng, T, E, K, p_pad=0.0, p_dup=0.0):
    tk = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32) if K <= E else \
        rng.integers(0, E, size=(T, K)).astype(np.int32)
    if p_pad:
        tk[rng.random((T, K)) < p_pad] = -1
    if p_dup and K > 1:
        for t in range(T):
            if rng.random() < p_dup:
                tk[t, 1] = tk[t, 0]
    return tk


def _rand_map(rng, E, R, contiguous):
    if contiguous:
        return (np.arange(E) // max(E // R, 1)).clip(0, R - 1).astype(np.int32)
    return rng.integers(0, R, size=E).astype(np.int32)


CASES = [  # (T, E, R, K, contiguous, p_pad, p_dup)
    (1, 4, 2, 1, True, 0.0, 0.0),
    (37, 16, 8, 2, True, 0.0, 0.0),
    (64, 12, 5, 3, False, 0.2, 0.3),
    (50, 256, 256, 8, True, 0.1, 0.0),
    (40, 200, 130, 6, False, 0.0, 0.2),
    (25, 8, 70, 4, False, 0.5, 0.0),
]


# ---------------------------------------------------------------- paper arithmetic
def test_paper_printed_arithmetic(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "paper_arithmetic.json")))
    d = g["destination_sets_ep64_top8"]
    assert math.comb(d["n"], d["k"]) == 4426165368 > d["lower_bound"]
    e = g["eid_metadata"]
    assert e["bits_per_destination"] * e["destinations"] // 8 == e["bytes"] == 128
    b = g["bitmap_metadata"]
    assert b["bits"] // 8 == b["bytes"] == 8
    o = g["in_payload_bitmap_overhead"]
    pct = 100.0 * (o["bitmap_bits"] / 8) / o["payload_bytes"]
    assert pct == 3.125 and abs(pct - o["printed_percent"]) < 0.01
    # the descriptor's bitmap is 4 x 64 bit: 32 B covers 256 ranks
    assert ref.DESC.fields["mask"][0].itemsize == 32


# ---------------------------------------------------------------- S1 masks
@pytest.mark.parametrize("case", CASES)
def test_masks_brute_force(case):
    T, E, R, K, contig, p_pad, p_dup = case
    rng = np.random.default_rng(hash(case) & 0xFFFF)
    e2r = _rand_map(rng, E, R, contig)
    tk = _rand_topk(rng, T, E, K, p_pad, p_dup)
    m = ref.masks(tk, e2r, R)
    for t in range(T):
        assert words_to_int(m[t]) == mask_int(tk[t], e2r)
        assert bin(words_to_int(m[t])).count("1") <= min(K, R)
        assert words_to_int(m[t]) >> R == 0
    # the order of ids inside a token does not matter
    tk2 = np.stack([rng.permutation(row) for row in tk]).astype(np.int32)
    assert np.array_equal(ref.masks(tk2, e2r, R), m)


def test_mask_bit_positions_every_rank():
    # one token per rank: expert r on rank r -> exactly bit r (word r // 64, bit r % 64)
    R = 256
    e2r = np.arange(R, dtype=np.int32)
    tk = np.arange(R, dtype=np.int32).reshape(R, 1)
    m = ref.masks(tk, e2r, R)
    for r in range(R):
        expect = [0, 0, 0, 0]
        expect[r // 64] = 1 << (r % 64)
        assert [int(v) for v in m[r]] == expect


def test_expected_popcount_closed_form():
    # uniform top-K without replacement, contiguous map, L experts per rank:
    # E[|destination set|] = R * (1 - C(E-L, K) / C(E, K))
    w = W.scaled(W.C0, n_tokens=20000)
    tk = W.topk_ids(w, 7, 0)
    m = ref.masks(tk, W.expert_to_rank(w), w.n_ranks)
    pc = np.array([bin(words_to_int(r)).count("1") for r in m])
    expect = 8 * (1 - math.comb(14, 2) / math.comb(16, 2))
    assert abs(expect - (2 - 1 / 15)) < 1e-12
    sd = math.sqrt((1 / 15) * (14 / 15) / len(pc))
    assert abs(pc.mean() - expect) < 5 * sd


def test_one_expert_per_rank_gives_exactly_k_destinations():
    w = W.scaled(W.C3, n_tokens=300)
    tk = W.topk_ids(w, 3, 5)
    _, _, desc, st = ref.plan(tk, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    assert (desc["n_dest"] == w.top_k).all()
    assert int(st["unicast_bytes"]) == w.top_k * int(st["multicast_bytes"])   # saved = 1 - 1/K exactly


# ---------------------------------------------------------------- S2/S3 plan
@pytest.mark.parametrize("case", CASES)
def test_plan_brute_force(case):
    T, E, R, K, contig, p_pad, p_dup = case
    rng = np.random.default_rng((hash(case) >> 3) & 0xFFFF)
    e2r = _rand_map(rng, E, R, contig)
    tk = _rand_topk(rng, T, E, K, p_pad, p_dup)
    rb = 48
    m, perm, desc, st = ref.plan(tk, e2r, R, rb)
    masks, perm_b, groups_b = plan_brute(tk, e2r)
    assert perm.tolist() == perm_b
    assert len(desc) == len(groups_b) == int(st["n_groups"])
    for d, g in zip(desc, groups_b):
        assert (words_to_int(d["mask"]), int(d["row_offset"]), int(d["row_count"]), int(d["n_dest"])) == g
        assert int(d["reserved0"]) == 0
    # invariants
    N = len(perm)
    assert int(st["n_rows"]) == N == sum(1 for x in masks if x)
    assert sorted(perm.tolist()) == [t for t in range(T) if masks[t]]
    assert int(desc["row_count"].sum()) == N if N else len(desc) == 0
    assert np.array_equal(desc["row_offset"], np.concatenate([[0], np.cumsum(desc["row_count"])[:-1]]))
    ints = [words_to_int(d["mask"]) for d in desc]
    assert all(a < b for a, b in zip(ints, ints[1:]))
    # accounting: one injected copy per row vs one per destination (Section 1)
    total_dest = sum(len(dest_set(tk[t], e2r)) for t in range(T))
    assert int(st["multicast_bytes"]) == N * rb
    assert int(st["unicast_bytes"]) == total_dest * rb
    rpd = [sum(1 for t in range(T) if r in dest_set(tk[t], e2r)) for r in range(256)]
    assert st["rows_per_dest"].tolist() == rpd
    assert sum(rpd) == total_dest
    mc, uc, rpd2 = ref.accounting_plain(tk, e2r, R, rb)
    assert (mc, uc, rpd2.tolist()) == (N * rb, total_dest * rb, rpd)


def test_all_equal_masks_is_identity_and_memcpy():
    rng = np.random.default_rng(11)
    T, E, R, K = 33, 8, 4, 2
    e2r = (np.arange(E) // 2).astype(np.int32)
    tk = np.tile(np.array([[5, 0]], dtype=np.int32), (T, 1))
    x = rng.integers(0, 2 ** 16, size=(T, 40), dtype=np.uint16)
    _, perm, desc, st = ref.plan(tk, e2r, R, 80)
    assert len(desc) == 1 and int(desc[0]["row_count"]) == T and perm.tolist() == list(range(T))
    packed, src, rtk = ref.pack(x, None, tk, perm)
    assert packed.tobytes() == x.tobytes()
    assert src.tolist() == list(range(T)) and np.array_equal(rtk, tk)


def test_k1_is_plain_alltoallv_stable_sort():
    # one destination per token (Section 4.3.3 rule 2): the plan is the textbook
    # stable counting sort by destination rank, and multicast saves nothing
    rng = np.random.default_rng(5)
    T, E, R = 500, 32, 16
    e2r = rng.integers(0, R, size=E).astype(np.int32)
    tk = rng.integers(0, E, size=(T, 1)).astype(np.int32)
    _, perm, desc, st = ref.plan(tk, e2r, R, 64)
    dest = e2r[tk[:, 0]]
    assert np.array_equal(perm, np.argsort(dest, kind="stable"))
    counts = np.bincount(dest, minlength=R)
    assert desc["row_count"].tolist() == counts[counts > 0].tolist()
    assert [int(np.log2(int(d["mask"][0]))) for d in desc] == np.nonzero(counts)[0].tolist()
    assert int(st["multicast_bytes"]) == int(st["unicast_bytes"]) == T * 64


def test_empty_and_padding_tokens():
    e2r = np.arange(4, dtype=np.int32)
    tk = np.array([[-1, -1], [2, -1], [-1, -1], [-1, 1]], dtype=np.int32)
    m, perm, desc, st = ref.plan(tk, e2r, 4, 16)
    assert perm.tolist() == [3, 1] and int(st["n_rows"]) == 2 and int(st["n_groups"]) == 2
    m, perm, desc, st = ref.plan(np.zeros((0, 2), np.int32), e2r, 4, 16)
    assert len(perm) == 0 and len(desc) == 0 and int(st["unicast_bytes"]) == 0


def test_invalid_expert_id_is_an_error():
    e2r = np.arange(4, dtype=np.int32)
    for bad in (4, -2, 1000):
        with pytest.raises(ref.OracleError) as ei:
            ref.plan(np.array([[0, bad]], dtype=np.int32), e2r, 4, 16)
        assert ei.value.code == ref.ERR_EXPERT
    with pytest.raises(ref.OracleError):
        ref.plan(np.array([[0, 1]], dtype=np.int32), e2r, 257, 16)


# ---------------------------------------------------------------- S4 pack
@pytest.mark.parametrize("fmt", ["bf16", "fp8"])
def test_pack_rows_meta_and_exactly_once(fmt):
    w = W.scaled(W.C0 if fmt == "bf16" else W.DispatchWorkload("t", 9, 8, 16, 2, 96, 256, "fp8", "uniform"),
                 n_tokens=96)
    tk = W.topk_ids(w, 2, 1)
    tk[5] = -1
    e2r = W.expert_to_rank(w)
    x, sc = W.payload_rows(w, 2, 1)
    _, perm, desc, st = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    packed, src, rtk = ref.pack(x, sc, tk, perm)
    assert packed.shape == (len(perm), w.row_bytes)
    xb = x.view(np.uint8).reshape(len(x), -1)
    for i, t in enumerate(perm):
        assert packed[i, :xb.shape[1]].tobytes() == xb[t].tobytes()
        if sc is not None:   # e4m3 codes first, then the fp32 scales
            assert packed[i, xb.shape[1]:].tobytes() == sc[t].tobytes()
            assert xb.shape[1] == w.hidden and packed.shape[1] == w.hidden + 4 * (w.hidden // 128)
        assert src[i] == t and rtk[i].tolist() == tk[t].tolist()
    # every (token, destination rank) pair is delivered exactly once
    for r in range(w.n_ranks):
        got = []
        for d in desc:
            if (words_to_int(d["mask"]) >> r) & 1:
                got += src[int(d["row_offset"]):int(d["row_offset"]) + int(d["row_count"])].tolist()
        want = [t for t in range(w.n_tokens) if r in dest_set(tk[t], e2r)]
        assert sorted(got) == want and len(got) == len(set(got))
        assert len(want) == int(st["rows_per_dest"][r])


# ---------------------------------------------------------------- deliver + unpack
def _peer_buffers(w, seed, my_rank, full=False, tweak=None):
    e2r = W.expert_to_rank(w)
    toks, bufs = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, seed, p)
        if tweak:
            tweak(p, tk)
        x, sc = W.payload_rows(w, seed, p)
        _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        packed, src, rtk = ref.pack(x, sc, tk, perm)
        bufs.append((desc, packed, src, rtk) if full else ref.deliver(desc, packed, src, rtk, my_rank))
        toks.append((tk, x, sc))
    return e2r, toks, bufs


def _xs_bytes(w):
    xrb = 2 * w.hidden if w.row_format == "bf16" else w.hidden
    return xrb, w.row_bytes - xrb


@pytest.mark.parametrize("fmt,my_rank", [("bf16", 0), ("bf16", 5), ("fp8", 3)])
def test_tier2_equals_tier1_equals_brute_force(fmt, my_rank):
    w = W.DispatchWorkload("t", 21, 8, 16, 2, 40, 128, fmt, "uniform")

    def tweak(p, tk):
        tk[3] = -1                 # a token with no expert
        tk[7, 1] = tk[7, 0]        # duplicate id inside a token: delivered once
        if p == 2:
            tk[:] = -1             # a peer that sends nothing

    e2r, toks, bufs = _peer_buffers(w, 4, my_rank, tweak=tweak)
    xrb, srb = _xs_bytes(w)
    cap = w.n_ranks * w.n_tokens * 2
    o2 = ref.unpack(bufs, w.top_k, e2r, my_rank, xrb, srb, cap)
    o1 = ref.dispatch_plain(toks, e2r, my_rank, cap)
    entries, offsets, rows, scales = dispatch_plain_brute(toks, e2r, my_rank)
    for a, b in zip(o2[:5], o1):
        assert (a is None and b is None) or np.array_equal(a, b)
    assert o1[4].tolist() == offsets
    assert list(zip(o1[2].tolist(), o1[3].tolist())) == entries
    assert [r.tobytes() for r in o1[0]] == rows
    if scales is not None:
        assert [r.tobytes() for r in o1[1]] == scales
    # inside an expert: strictly increasing (peer, token)
    for le in range(len(offsets) - 1):
        seg = entries[offsets[le]:offsets[le + 1]]
        assert all(a < b for a, b in zip(seg, seg[1:]))
    # rows addressed to this rank
    assert o2[5] == sum(1 for tk, _, _ in toks for t in range(len(tk)) if my_rank in dest_set(tk[t], e2r))
    # a sender's complete buffer is accepted too: groups without our bit are skipped
    _, _, full = _peer_buffers(w, 4, my_rank, full=True, tweak=tweak)
    o3 = ref.unpack(full, w.top_k, e2r, my_rank, xrb, srb, cap)
    for a, b in zip(o3, o2):
        assert (a is None and b is None) or np.array_equal(a, b)


def test_deliver_keeps_exactly_the_groups_naming_the_rank():
    w = W.scaled(W.C0, n_tokens=64)
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, 9, 3)
    x, _ = W.payload_rows(w, 9, 3)
    _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    packed, src, rtk = ref.pack(x, None, tk, perm)
    for r in range(w.n_ranks):
        d2, r2, s2, t2 = ref.deliver(desc, packed, src, rtk, r)
        keep = [i for i, t in enumerate(perm) if r in dest_set(tk[t], e2r)]
        assert s2.tolist() == perm[keep].tolist()
        assert r2.tobytes() == packed[keep].tobytes() and np.array_equal(t2, rtk[keep])
        assert all((words_to_int(d["mask"]) >> r) & 1 for d in d2)
        assert np.array_equal(d2["row_offset"], np.concatenate([[0], np.cumsum(d2["row_count"])[:-1]]).astype(np.uint32))
        # bitmaps travel unchanged
        sent = {words_to_int(d["mask"]) for d in desc if (words_to_int(d["mask"]) >> r) & 1}
        assert {words_to_int(d["mask"]) for d in d2} == sent


def test_unpack_errors():
    w = W.scaled(W.C0, n_tokens=16)
    e2r, toks, bufs = _peer_buffers(w, 1, 0)
    xrb, srb = _xs_bytes(w)
    with pytest.raises(ref.OracleError) as ei:
        ref.unpack(bufs, w.top_k, e2r, 0, xrb, srb, 1)
    assert ei.value.code == ref.ERR_CAPACITY
    d, r, s, t = bufs[0]
    if len(d):
        d = d.copy(); d["row_count"][-1] += 5
        with pytest.raises(ref.OracleError) as ei:
            ref.unpack([(d, r, s, t)], w.top_k, e2r, 0, xrb, srb, 1000)
        assert ei.value.code == ref.ERR_INPUT


def test_hand_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "hand_worked_dispatch.json")))
    R, E, K = g["n_ranks"], g["n_experts"], g["top_k"]
    e2r = (np.arange(E) // 2).astype(np.int32)
    tk = np.array(g["topk"], dtype=np.int32)
    rb = 32
    x = (np.arange(len(tk) * 16, dtype=np.uint16) * 7 + 1).reshape(len(tk), 16)
    m, perm, desc, st = ref.plan(tk, e2r, R, rb)
    assert m[:, 0].tolist() == g["mask_word0"] and not m[:, 1:].any()
    assert perm.tolist() == g["perm"]
    assert [dict(mask=int(d["mask"][0]), row_offset=int(d["row_offset"]), row_count=int(d["row_count"]),
                 n_dest=int(d["n_dest"])) for d in desc] == g["groups"]
    assert int(st["multicast_bytes"]) == g["multicast_rows"] * rb
    assert int(st["unicast_bytes"]) == g["unicast_rows"] * rb
    assert st["rows_per_dest"][:R].tolist() == g["rows_per_dest"] and not st["rows_per_dest"][R:].any()
    packed, src, rtk = ref.pack(x, None, tk, perm)
    buf = ref.deliver(desc, packed, src, rtk, 0)
    assert buf[2].tolist() == g["delivered_to_rank0_src_tokens"]
    o = ref.unpack([buf], K, e2r, 0, rb, 0, 16)
    assert o[4].tolist() == g["rank0_single_peer"]["expert_offsets"]
    assert o[3].tolist() == g["rank0_single_peer"]["src_token"]
    assert o[0].tobytes() == x[g["rank0_single_peer"]["src_token"]].tobytes()
    o = ref.unpack([buf, buf], K, e2r, 0, rb, 0, 16)
    assert o[4].tolist() == g["rank0_two_identical_peers"]["expert_offsets"]
    assert o[2].tolist() == g["rank0_two_identical_peers"]["src_peer"]
    assert o[3].tolist() == g["rank0_two_identical_peers"]["src_token"]


# ---------------------------------------------------------------- AllGather
def test_allgather_is_concatenation_and_a_dispatch_special_case(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "paper_arithmetic.json")))
    w = W.AllGatherWorkload("ag", 40, 8, 1024)
    shards = [W.allgather_shard(w, 3, r) for r in range(w.n_ranks)]
    d, st = ref.plan_allgather(w.n_ranks, w.shard_bytes)
    assert words_to_int(d[0]["mask"]) == (1 << w.n_ranks) - 1 and int(d[0]["row_count"]) == 1
    assert int(d[0]["n_dest"]) == w.n_ranks
    # unicast would inject R copies (R - 1 = 7 to the other nodes, Section 2.3.1, plus this rank's own)
    assert int(st["unicast_bytes"]) == w.n_ranks * int(st["multicast_bytes"])
    assert w.n_ranks - 1 == g["unicast_copies_allgather_8"]["copies"]
    assert ref.pack_allgather(shards[2]).tobytes() == shards[2].tobytes()
    out = ref.unpack_allgather(shards)
    assert out.tobytes() == np.concatenate(shards).tobytes()
    # the same thing as a dispatch: one token per rank naming every rank's expert
    R = w.n_ranks
    e2r = np.arange(R, dtype=np.int32)
    tk = np.arange(R, dtype=np.int32).reshape(1, R)
    bufs = []
    for p in range(R):
        _, perm, desc, st2 = ref.plan(tk, e2r, R, w.shard_bytes)
        assert desc.tobytes() == d.tobytes()
        for f in ("n_rows", "n_groups", "multicast_bytes", "unicast_bytes"):
            assert int(st2[f]) == int(st[f])
        assert np.array_equal(st2["rows_per_dest"], st["rows_per_dest"])
        packed, src, rtk = ref.pack(shards[p].reshape(1, -1), None, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, 5))
    o = ref.unpack(bufs, R, e2r, 5, w.shard_bytes, 0, R)
    assert o[0].tobytes() == out.tobytes()


def test_allgather_bytes_saved_128_ranks():
    _, st = ref.plan_allgather(128, 2 << 20)
    assert 1 - int(st["multicast_bytes"]) / int(st["unicast_bytes"]) == 1 - 1 / 128


# ---------------------------------------------------------------- workloads (structure the configs promise)
def test_workload_structure():
    tk = W.topk_ids(W.scaled(W.C1, n_tokens=256), 1, 3)
    assert tk.shape == (256, 8) and all(len(set(r)) == 8 for r in tk.tolist())
    nodes = (W.expert_to_rank(W.C1)[tk] // 8)
    assert max(len(set(r)) for r in nodes.tolist()) <= 4          # group-limited routing
    tk3 = W.topk_ids(W.scaled(W.C3, n_tokens=256), 1, 0)
    assert all(len(set(r)) == 8 for r in tk3.tolist())
    order = W.zipf_order(W.C3, 1)
    assert sorted(order.tolist()) == list(range(256))
    hot = (tk3 == order[0]).any(axis=1).mean()
    assert hot > 0.5                                              # the hottest expert is in most tokens
    assert np.array_equal(W.topk_ids(W.C0, 1, 2), W.topk_ids(W.C0, 1, 2))
    assert not np.array_equal(W.topk_ids(W.C0, 1, 2), W.topk_ids(W.C0, 1, 3))
    x, _ = W.payload_rows(W.C0, 1, 0, np.array([5, 9]))
    xa, _ = W.payload_rows(W.C0, 1, 0)
    assert np.array_equal(x, xa[[5, 9]])                          # rows can be drawn lazily
    q, s = W.payload_rows(W.scaled(W.C2, n_tokens=4), 1, 0)
    assert q.dtype == np.uint8 and q.shape == (4, 7168) and s.shape == (4, 56)
    assert ((q & 0x7F) != 0x7F).all() and ((q & 0x7F) == 0x7E).any(axis=1).all()   # no NaN; amax hits 448
