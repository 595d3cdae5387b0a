"""GPU parity of the relay step (mw_set_forwarding, mw_relay) against the CPU oracle:
every child's descriptors, rows and metadata and the copy accounting, bit-exact; plus the
end-to-end property that delivery through relays equals direct delivery."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_22428_amd import binding as B
from paper_2605_22428_amd import workloads as W

import gpu_harness as H

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _ctx(w, my_rank, max_hops, max_tokens=None, max_recv_rows=None, row_stride=0):
    return B.Context(w.n_ranks, w.n_experts, w.top_k, my_rank, w.hidden, H.fmt_code(w),
                     max_tokens if max_tokens is not None else w.n_tokens,
                     max_recv_rows if max_recv_rows is not None else w.n_ranks * w.n_tokens,
                     W.expert_to_rank(w), device=H.DEV, max_hops=max_hops, row_stride=row_stride)


def _in_record(rec):
    """One mw_recv_peer record on the device for a dict of device tensors."""
    return B.peers_table([rec], H.DEV)


def gpu_relay(ctx, rec, next_hop, n_hops, capacity):
    ctx.mw_set_forwarding(next_hop, n_hops)
    ch = B.RelayChildren(ctx, n_hops, capacity)
    table = _in_record(rec)
    ctx.mw_relay(table, ch.table, capacity, ch.stats)
    st = ctx.mw_get_relay_stats(ch.stats)
    return ch, st, table


def child_host(ch, st, h, row_bytes=None):
    g, n = int(st["groups_per_hop"][h]), int(st["rows_per_hop"][h])
    rb = ch.rows[h].shape[1] if row_bytes is None else row_bytes
    return (H.host(ch.desc[h]).reshape(-1).view(B.DESC_DTYPE)[:g], H.host(ch.rows[h])[:n, :rb],
            H.host(ch.row_src_token[h])[:n], H.host(ch.row_topk[h])[:n])


def check_children(ch, st, parent_host, next_hop, n_hops, row_bytes, hops=None):
    desc, rows, src, rtk = parent_host
    for h in (range(n_hops) if hops is None else hops):
        want = ref.relay_child(desc, rows, src, rtk, next_hop, n_hops, h)
        got = child_host(ch, st, h, row_bytes)
        H.assert_same_bytes(got[0].view(np.uint8), want[0].view(np.uint8), "child %d desc" % h)
        H.assert_same_bytes(got[1], want[1], "child %d rows" % h)
        H.assert_same_bytes(got[2], want[2], "child %d src_token" % h)
        H.assert_same_bytes(got[3], want[3], "child %d row_topk" % h)
    fwd, uni, rph = ref.relay_accounting(desc, row_bytes, next_hop, n_hops)
    assert int(st["error_flags"]) == 0
    assert int(st["forward_bytes"]) == fwd and int(st["unicast_bytes"]) == uni
    assert st["rows_per_hop"][:n_hops].tolist() == rph.tolist()
    assert int(st["n_groups_in"]) == len(desc) and int(st["n_rows_in"]) == len(rows)
    assert not st["rows_per_hop"][n_hops:].any() and not st["groups_per_hop"][n_hops:].any()


def _send(ctx, w, seed, p):
    tk = W.topk_ids(w, seed, p)
    x, sc = W.payload_rows(w, seed, p)
    g = H.GpuSend(ctx, tk, x, sc)
    return tk, x, sc, g


def _two_server_tables(n_per):
    R = 2 * n_per
    out = []
    for s in range(R):
        t = np.empty(R, dtype=np.int32)
        for r in range(R):
            t[r] = (r % n_per) if r // n_per == s // n_per else n_per
        out.append(t)
    return out, n_per + 1


@pytest.mark.parametrize("fmt,seed", [("bf16", 1), ("bf16", 2), ("fp8", 3)])
def test_relay_children_match_oracle_random_tables(fmt, seed):
    hidden = 1024
    w = W.scaled(W.C1 if fmt == "bf16" else W.C2, n_tokens=333, hidden=hidden)
    _say("relay random table", w.name, "seed", seed)
    rng = np.random.default_rng(seed)
    n_hops = [5, 17, 64][seed - 1]
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    ctx = _ctx(w, 0, 64)
    tk, x, sc, g = _send(ctx, w, seed, 0)
    H.check_send(w, g, tk, x, sc)
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, n_hops, w.n_tokens)
    parent = H.oracle_send(w, tk, x, sc)
    check_children(ch, st, parent, next_hop, n_hops, w.row_bytes)
    ctx.close()


def test_relay_identity_and_single_hop_tables():
    w = W.scaled(W.C1, n_tokens=130, hidden=512)
    ctx = _ctx(w, 0, 64)
    tk, x, sc, g = _send(ctx, w, 1, 0)
    parent = H.oracle_send(w, tk, x, sc)
    ident = np.arange(w.n_ranks, dtype=np.int32)
    ch, st, _ = gpu_relay(ctx, g.full_record(), ident, w.n_ranks, w.n_tokens)
    check_children(ch, st, parent, ident, w.n_ranks, w.row_bytes)
    assert int(st["forward_bytes"]) == int(st["unicast_bytes"]) == int(g.stats["unicast_bytes"])
    one = np.zeros(w.n_ranks, dtype=np.int32)
    ch, st, _ = gpu_relay(ctx, g.full_record(), one, 1, w.n_tokens)
    got = child_host(ch, st, 0)
    H.assert_same_bytes(got[0].view(np.uint8), parent[0].view(np.uint8), "one hop desc")
    H.assert_same_bytes(got[1], parent[1], "one hop rows")
    assert int(st["forward_bytes"]) == int(g.stats["multicast_bytes"])
    ctx.close()


def test_relay_all_equal_bitmaps_one_long_group():
    # every token to the same two ranks: one group of 700 rows, row -> group mapping spans tiles
    R, E, K, T, Hh = 8, 8, 2, 700, 256
    w = W.DispatchWorkload("same", 51, R, E, K, T, Hh, "bf16", "uniform")
    tk = np.tile(np.array([[2, 5]], dtype=np.int32), (T, 1))
    x, _ = W.payload_rows(w, 1, 0)
    ctx = _ctx(w, 0, 8)
    g = H.GpuSend(ctx, tk, x, None)
    assert g.G == 1 and g.N == T
    next_hop = np.array([0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32)
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, 4, T)
    check_children(ch, st, H.oracle_send(w, tk, x, None), next_hop, 4, w.row_bytes)
    assert st["rows_per_hop"][:4].tolist() == [0, T, T, 0]
    ctx.close()


def test_delivery_through_relays_equals_direct_delivery_on_gpu():
    """Section 3.2's two-server topology, everything on the GPU: source -> (same-index relay of
    the other server) -> destination, then mw_unpack; equals the plain definition."""
    n_per = 4
    w = W.DispatchWorkload("t2s", 52, 2 * n_per, 16, 3, 96, 512, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tables, n_hops = _two_server_tables(n_per)
    d = 5
    ctx = _ctx(w, d, n_hops)
    toks, recs, keep = [], [], []
    for p in range(w.n_ranks):
        tk, x, sc, g = _send(ctx, w, 3, p)
        toks.append((tk, x, sc))
        ch, st, _ = gpu_relay(ctx, g.full_record(), tables[p], n_hops, w.n_tokens)
        if p // n_per == d // n_per:
            h = d % n_per
        else:
            h = n_per
            relay = (p % n_per) + (d // n_per) * n_per
            rec1 = ch.record(h, int(st["groups_per_hop"][h]), int(st["rows_per_hop"][h]))
            ch2, st2, _ = gpu_relay(ctx, rec1, tables[relay], n_hops, w.n_tokens)
            keep.append((ch, g))
            ch, st, h = ch2, st2, d % n_per
        assert int(st["error_flags"]) == 0
        recs.append(H.shrink(ch.record(h, int(st["groups_per_hop"][h]), int(st["rows_per_hop"][h]))))
        keep.append((ch, g))
    cap = sum(r["n_rows"] for r in recs) * 2
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, ref.dispatch_plain(toks, e2r, d, cap), "through relays")
    ctx.close()


def test_relay_capacity_bad_descriptors_and_host_errors():
    w = W.scaled(W.C1, n_tokens=200, hidden=256)
    ctx = _ctx(w, 0, 16)
    tk, x, sc, g = _send(ctx, w, 1, 0)
    next_hop = (np.arange(w.n_ranks) % 3).astype(np.int32)
    # no forwarding table yet
    ch = B.RelayChildren(ctx, 3, 10)
    with pytest.raises(B.MwError):
        ctx.mw_relay(_in_record(g.full_record()), ch.table, 10, ch.stats)
    with pytest.raises(B.MwError):
        ctx.mw_set_forwarding(next_hop, 17)                      # more hops than the context allows
    with pytest.raises(B.MwError):
        ctx.mw_set_forwarding(np.full(w.n_ranks, 5, dtype=np.int32), 3)   # entry outside [0, n_hops)
    # children too small: flagged, and what was written is a prefix of the oracle's child
    cap = 50
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, 3, cap)
    assert int(st["error_flags"]) & B.MW_FLAG_OUT_CAPACITY
    parent = H.oracle_send(w, tk, x, sc)
    for h in range(3):
        want = ref.relay_child(*parent, next_hop, 3, h)
        gg, n = int(st["groups_per_hop"][h]), int(st["rows_per_hop"][h])
        assert n <= cap and n < len(want[1])
        got = child_host(ch, st, h)
        H.assert_same_bytes(got[0].view(np.uint8), want[0][:gg].view(np.uint8), "prefix desc")
        H.assert_same_bytes(got[1], want[1][:n], "prefix rows")
    assert int(st["forward_bytes"]) == w.row_bytes * int(st["rows_per_hop"][:3].sum())
    # dropped: a descriptor reaching outside the buffer (3), its successor, which now starts
    # inside the range 3 claims (4), and one overlapping its predecessor (7)
    desc = parent[0].copy()
    desc["row_count"][3] += 1000
    desc["row_offset"][7] -= 1
    rec = g.full_record()
    rec = dict(rec, desc=H.dev(desc.view(np.uint8).reshape(-1, B.DESC_BYTES)))
    ch, st, _ = gpu_relay(ctx, rec, next_hop, 3, w.n_tokens)
    assert int(st["error_flags"]) & B.MW_FLAG_BAD_DESC
    assert int(st["n_groups_in"]) == len(desc) - 3
    good = np.delete(desc, [3, 4, 7])
    fwd, uni, rph = ref.relay_accounting(good, w.row_bytes, next_hop, 3)
    assert st["rows_per_hop"][:3].tolist() == rph.tolist() and int(st["unicast_bytes"]) == uni
    # a bitmap that names a rank this configuration does not have: that bit is forwarded nowhere
    # and flagged, everything else is as without it
    desc = parent[0].copy()
    desc["mask"][5][1] |= np.uint64(1) << np.uint64(3)            # rank 67 of 64
    desc["mask"][6][2] |= np.uint64(1)                            # rank 128
    rec = dict(g.full_record(), desc=H.dev(desc.view(np.uint8).reshape(-1, B.DESC_BYTES)))
    ch, st, _ = gpu_relay(ctx, rec, next_hop, 3, w.n_tokens)
    assert int(st["error_flags"]) == B.MW_FLAG_BAD_RANK
    for h in range(3):
        want = ref.relay_child(*parent, next_hop, 3, h)
        got = child_host(ch, st, h)
        H.assert_same_bytes(got[0].view(np.uint8), want[0].view(np.uint8), "child %d desc without the bad bits" % h)
        H.assert_same_bytes(got[1], want[1], "child %d rows" % h)
    fwd, uni, rph = ref.relay_accounting(parent[0], w.row_bytes, next_hop, 3)
    assert (int(st["forward_bytes"]), int(st["unicast_bytes"])) == (fwd, uni)
    with pytest.raises(ref.OracleError):
        ref.relay_child(desc, *parent[1:], next_hop, 3, 0)
    # the flag word is cleared again: a clean relay afterwards reports no error
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, 3, w.n_tokens)
    assert int(st["error_flags"]) == 0
    ctx.close()


def test_relay_full_size_c1_two_level_topology():
    """C1 at full size: 64 ranks = 8 servers x 8; rank 0's forwarding table has 8 direct hops
    and one hop per remote server (its same-index device)."""
    w = W.C1
    n_per, n_srv = 8, 8
    next_hop = np.array([(r % n_per) if r // n_per == 0 else n_per + (r // n_per) - 1 for r in range(w.n_ranks)],
                        dtype=np.int32)
    n_hops = n_per + n_srv - 1
    ctx = _ctx(w, 0, 16, max_recv_rows=1)
    tk = W.topk_ids(w, W.BASE_SEED, 0)
    tokens = np.arange(0, w.n_tokens, 5)
    x, _ = W.payload_full(w, W.BASE_SEED, 0, tokens)
    g = H.GpuSend(ctx, tk, x, None)
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, n_hops, w.n_tokens)
    parent = H.oracle_send(w, tk, x, None)
    check_children(ch, st, parent, next_hop, n_hops, w.row_bytes, hops=(0, 7, 8, 14))
    saved = 1.0 - int(st["forward_bytes"]) / int(st["unicast_bytes"])
    _say("  copies per token", int(st["forward_bytes"]) / w.row_bytes / g.N, "saved vs unicast", round(saved, 4))
    ctx.close()


@pytest.mark.parametrize("hidden", [5128, 5184, 8200])
def test_relay_long_rows(hidden):
    """Rows of 641, 648 and 1025 chunks: the relay's row mover in each of its launch shapes."""
    w = W.DispatchWorkload("relay_rows", 93, 16, 32, 4, 90, hidden, "bf16", "uniform")
    next_hop = (np.arange(w.n_ranks) % 5).astype(np.int32)
    ctx = _ctx(w, 3, 8)
    tk, x, sc, g = _send(ctx, w, 2, 3)
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, 5, w.n_tokens)
    check_children(ch, st, H.oracle_send(w, tk, x, sc), next_hop, 5, w.row_bytes)
    ctx.close()


@pytest.mark.parametrize("fmt", ["bf16", "fp8"])
def test_relay_with_a_row_stride(fmt):
    """Rows a stride apart on both sides of the relay (parent buffer and every child's)."""
    w = W.scaled(W.C1 if fmt == "bf16" else W.C2, n_tokens=210, hidden=1024)
    stride = (w.row_bytes + 127) // 128 * 128 + 128
    next_hop = (np.arange(w.n_ranks) % 6).astype(np.int32)
    ctx = _ctx(w, 7, 8, row_stride=stride)
    tk, x, sc, g = _send(ctx, w, 4, 7)
    H.check_send(w, g, tk, x, sc)
    ch, st, _ = gpu_relay(ctx, g.full_record(), next_hop, 6, w.n_tokens)
    check_children(ch, st, H.oracle_send(w, tk, x, sc), next_hop, 6, w.row_bytes)
    for h in range(6):
        n = int(st["rows_per_hop"][h])
        assert not H.host(ch.rows[h])[:n, w.row_bytes:].any(), "bytes between a child's rows were written"
    ctx.close()


@pytest.mark.parametrize("which", ["bf16_short_rows", "bf16_long_rows", "bf16_single_waves", "fp8"])
def test_relay_stream_index_of_the_next_buffer_rides_with_the_copy(which):
    """mw_relay_index + mw_relay_copy_index_next + mw_relay_copy over a stream of buffers on two
    contexts with different forwarding tables: every step's children and statistics against the
    oracle, whatever index ran beside its copy; one buffer is short and one is empty."""
    w = {"bf16_short_rows": W.scaled(W.C1, n_tokens=300, hidden=1024),
         "bf16_long_rows": W.scaled(W.C1, n_tokens=150, hidden=7168),      # three 320-lane workgroups per row
         "bf16_single_waves": W.scaled(W.C1, n_tokens=100, hidden=5184),   # 648 chunks: 64-lane workgroups
         "fp8": W.scaled(W.C2, n_tokens=260, hidden=1024)}[which]
    _say("relay stream", w.name)
    rng = np.random.default_rng(5)
    tables = [(rng.integers(0, 9, size=w.n_ranks).astype(np.int32), 9),
              (rng.integers(0, 33, size=w.n_ranks).astype(np.int32), 33)]
    ctxs = [_ctx(w, 0, 64), _ctx(w, 0, 64)]
    for c, (nh, n) in zip(ctxs, tables):
        c.mw_set_forwarding(nh, n)
    sizes = [w.n_tokens, 77, 0, w.n_tokens, 130]
    steps = []
    for i, T in enumerate(sizes):
        tk = W.topk_ids(w, 20 + i, i)[:T].copy()
        x, sc = W.payload_rows(w, 20 + i, i)
        x, sc = x[:T].copy(), (None if sc is None else sc[:T].copy())
        g = H.GpuSend(ctxs[0], tk, x, sc)
        nh, n = tables[i % 2]
        steps.append(dict(tk=tk, x=x, sc=sc, g=g, table=_in_record(g.full_record()),
                          ch=B.RelayChildren(ctxs[i % 2], n, w.n_tokens)))
    s0 = steps[0]
    ctxs[0].mw_relay_index(s0["table"], s0["ch"].table, w.n_tokens, s0["ch"].stats)
    for i, st in enumerate(steps):
        cur = ctxs[i % 2]
        if i + 1 < len(steps):
            nx = steps[i + 1]
            cur.mw_relay_copy_index_next(st["table"], st["ch"].table, st["ch"].stats, ctxs[(i + 1) % 2], nx["table"],
                                         nx["ch"].table, w.n_tokens, nx["ch"].stats)
        else:
            cur.mw_relay_copy(st["table"], st["ch"].table, st["ch"].stats)
    torch.cuda.synchronize()
    for i, st in enumerate(steps):
        nh, n = tables[i % 2]
        stats = ctxs[i % 2].mw_get_relay_stats(st["ch"].stats)
        parent = H.oracle_send(w, st["tk"], st["x"], st["sc"])
        check_children(st["ch"], stats, parent, nh, n, w.row_bytes)
    # argument errors: the same context twice, a missing next buffer
    with pytest.raises(B.MwError) as ei:
        ctxs[0].mw_relay_copy_index_next(s0["table"], s0["ch"].table, s0["ch"].stats, ctxs[0], s0["table"],
                                         s0["ch"].table, w.n_tokens, s0["ch"].stats)
    assert ei.value.status == B.MW_ERR_INVALID_ARG
    with pytest.raises(B.MwError) as ei:
        ctxs[0].mw_relay_copy_index_next(s0["table"], s0["ch"].table, s0["ch"].stats, ctxs[1], None,
                                         steps[1]["ch"].table, w.n_tokens, steps[1]["ch"].stats)
    assert ei.value.status == B.MW_ERR_INVALID_ARG
    for c in ctxs:
        c.close()


@pytest.mark.parametrize("which", ["bf16_long_rows", "fp8", "bf16_short_rows"])
def test_relay_batch_two_buffers_a_launch(which):
    """mw_relay_batch over a stream of seven buffers on four contexts with two forwarding tables: two
    copies and the next two indexes per launch, then a launch with one copy and no index; every
    buffer's children and statistics against the oracle.  One buffer is short, one is empty."""
    w = {"bf16_short_rows": W.scaled(W.C1, n_tokens=300, hidden=1024),
         "bf16_long_rows": W.scaled(W.C1, n_tokens=150, hidden=7168),
         "fp8": W.scaled(W.C2, n_tokens=260, hidden=1024)}[which]
    _say("relay batch", w.name)
    rng = np.random.default_rng(6)
    tables = [(rng.integers(0, 9, size=w.n_ranks).astype(np.int32), 9),
              (rng.integers(0, 33, size=w.n_ranks).astype(np.int32), 33)]
    ctxs = [_ctx(w, 0, 64) for _ in range(4)]
    for i, c in enumerate(ctxs):
        c.mw_set_forwarding(*tables[i % 2])
    sizes = [w.n_tokens, 77, 0, w.n_tokens, 130, w.n_tokens, 5]
    steps = []
    for i, T in enumerate(sizes):
        tk = W.topk_ids(w, 40 + i, i)[:T].copy()
        x, sc = W.payload_rows(w, 40 + i, i)
        x, sc = x[:T].copy(), (None if sc is None else sc[:T].copy())
        g = H.GpuSend(ctxs[0], tk, x, sc)
        c = ctxs[i % 4]
        ch = B.RelayChildren(c, tables[i % 2][1], w.n_tokens)
        table = _in_record(g.full_record())
        steps.append(dict(tk=tk, x=x, sc=sc, g=g, table=table, ch=ch, ctx=c,
                          job=B.relay_job(c, table, ch.table, w.n_tokens, ch.stats)))
    for st in steps[:2]:
        st["ctx"].mw_relay_index(st["table"], st["ch"].table, w.n_tokens, st["ch"].stats)
    B.mw_relay_batch([steps[0]["job"], steps[1]["job"]], [steps[2]["job"], steps[3]["job"]])
    B.mw_relay_batch([steps[2]["job"], steps[3]["job"]], [steps[4]["job"], steps[5]["job"]])
    B.mw_relay_batch([steps[4]["job"], steps[5]["job"]], [steps[6]["job"]])
    B.mw_relay_batch([steps[6]["job"]], [])
    torch.cuda.synchronize()
    for i, st in enumerate(steps):
        nh, n = tables[i % 2]
        stats = st["ctx"].mw_get_relay_stats(st["ch"].stats)
        check_children(st["ch"], stats, H.oracle_send(w, st["tk"], st["x"], st["sc"]), nh, n, w.row_bytes)
    # argument errors: a context twice, too many jobs, none to copy
    for bad in (([steps[0]["job"], steps[0]["job"]], []), ([steps[0]["job"]], [steps[0]["job"]]),
                ([s_["job"] for s_ in steps[:5]], []), ([], [steps[1]["job"]])):
        with pytest.raises(B.MwError) as ei:
            B.mw_relay_batch(*bad)
        assert ei.value.status == B.MW_ERR_INVALID_ARG
    for c in ctxs:
        c.close()


def _wide(n_ranks, n_experts, n_tokens=300, hidden=512):
    """A Zipf-routed workload over more than 64 ranks: bitmaps of two to four words."""
    import dataclasses
    return dataclasses.replace(W.C3, name="ep%d" % n_ranks, n_ranks=n_ranks, n_experts=n_experts,
                               n_tokens=n_tokens, hidden=hidden)


@pytest.mark.parametrize("n_ranks,n_experts,n_hops,keep", [(96, 192, 11, False), (128, 256, 40, True),
                                                            (200, 200, 7, False), (256, 256, 64, True),
                                                            (65, 130, 3, False)])
def test_relay_bitmaps_of_more_than_one_word(n_ranks, n_experts, n_hops, keep):
    """The index reads only the bitmap words that can name a rank (one, two or four): every width,
    with a last word that is partly used, in both forms of the metadata update, and the same
    index riding in a stream's copy launch."""
    w = _wide(n_ranks, n_experts)
    _say("relay over", n_ranks, "ranks,", n_hops, "hops, metadata kept:", keep)
    rng = np.random.default_rng(n_ranks)
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    next_hop[rng.integers(0, w.n_ranks, size=n_hops)] = np.arange(n_hops)      # every hop in use
    ctx = _ctx(w, 0, 64)
    ctx.mw_ctx_set_options(B.MW_OPT_RELAY_KEEP_METADATA if keep else 0)
    tk, x, sc, g = _send(ctx, w, 5, 0)
    parent = H.oracle_send(w, tk, x, sc)
    ch, st, table = gpu_relay(ctx, g.full_record(), next_hop, n_hops, w.n_tokens)

    def check(ch, st):
        for h in range(n_hops):
            want = ref.relay_child(*parent, next_hop, n_hops, h, update_metadata=not keep)
            got = child_host(ch, st, h, w.row_bytes)
            for a, b, what in zip(got, want, ("desc", "rows", "src_token", "row_topk")):
                H.assert_same_bytes(a.view(np.uint8), b.view(np.uint8), "child %d %s" % (h, what))
        fwd, uni, rph = ref.relay_accounting(parent[0], w.row_bytes, next_hop, n_hops)
        assert int(st["error_flags"]) == 0
        assert (int(st["forward_bytes"]), int(st["unicast_bytes"])) == (fwd, uni)
        assert st["rows_per_hop"][:n_hops].tolist() == rph.tolist()
        assert int(st["n_groups_in"]) == len(parent[0]) and int(st["n_rows_in"]) == len(parent[1])

    check(ch, st)
    # the same index as a rider: context 2 indexes in the launch that copies for context 1
    ctx2 = _ctx(w, 0, 64)
    ctx2.mw_ctx_set_options(B.MW_OPT_RELAY_KEEP_METADATA if keep else 0)
    ctx2.mw_set_forwarding(next_hop, n_hops)
    ch2 = B.RelayChildren(ctx2, n_hops, w.n_tokens)
    ctx.mw_relay_index(table, ch.table, w.n_tokens, ch.stats)
    ctx.mw_relay_copy_index_next(table, ch.table, ch.stats, ctx2, table, ch2.table, w.n_tokens, ch2.stats)
    ctx2.mw_relay_copy(table, ch2.table, ch2.stats)
    check(ch, ctx.mw_get_relay_stats(ch.stats))
    check(ch2, ctx2.mw_get_relay_stats(ch2.stats))
    # a bit for a rank that does not exist, in the last word that is partly used and beyond it
    if n_ranks % 64:
        bad = H.host(g.buf.desc).copy().reshape(-1).view(B.DESC_DTYPE)
        bad["mask"][1][n_ranks // 64] |= np.uint64(1) << np.uint64(n_ranks % 64)
        rec = dict(g.full_record()); rec["desc"] = H.dev(bad.view(np.uint8).reshape(-1, B.DESC_BYTES))
        ch3, st3, _ = gpu_relay(ctx, rec, next_hop, n_hops, w.n_tokens)
        assert int(st3["error_flags"]) & B.MW_FLAG_BAD_RANK
    ctx.close(); ctx2.close()
