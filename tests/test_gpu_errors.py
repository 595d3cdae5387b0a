"""Receive-side inputs that are inconsistent (a peer's metadata is whatever the peer wrote): the
kernels' own checks must turn each of them into an MW_FLAG_* bit, leave the offending item out,
deliver everything else exactly, and finish normally.  Expected outputs come from the oracle's
plain definition with the dropped (peer, token) pairs taken out of the input."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_22428_amd import binding as B
from paper_2605_22428_amd import workloads as W

import gpu_harness as H

pytestmark = pytest.mark.gpu

W_SMALL = W.DispatchWorkload("small", 31, 8, 16, 2, 96, 256, "bf16", "uniform")
MY_RANK = 3


def _regions(ctx, w=W_SMALL, seed=4, my_rank=MY_RANK):
    recs, toks = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, seed, p)
        x, _ = W.payload_rows(w, seed, p)
        g = H.GpuSend(ctx, tk, x, None)
        recs.append(H.shrink(g.deliver(my_rank)))
        toks.append((tk, x, None))
    return recs, toks


def _without(toks, dropped):
    """The plain definition's input with the given (peer, token) pairs going nowhere."""
    out = []
    for p, (tk, x, sc) in enumerate(toks):
        tk = tk.copy()
        for (pp, t) in dropped:
            if pp == p:
                tk[t] = -1
        out.append((tk, x, sc))
    return out


def _expect(gu, toks, dropped, flag, cap):
    e2r = W.expert_to_rank(W_SMALL)
    want = ref.dispatch_plain(_without(toks, dropped), e2r, MY_RANK, cap)
    assert int(gu.stats["error_flags"]) == flag, hex(int(gu.stats["error_flags"]))
    o = gu.host_out()
    H.assert_same_bytes(o[4], want[4], "expert_offsets")
    H.assert_same_bytes(o[2], want[2], "out_src_peer")
    H.assert_same_bytes(o[3], want[3], "out_src_token")
    H.assert_same_bytes(o[0], want[0], "out_rows")


def test_source_token_out_of_range_is_dropped():
    ctx = H.make_ctx(W_SMALL, MY_RANK)
    recs, toks = _regions(ctx)
    dropped = []
    for p, row, bad in ((1, 0, W_SMALL.n_tokens + 5), (4, 2, -3)):
        dropped.append((p, int(H.host(recs[p]["row_src_token"])[row])))
        recs[p]["row_src_token"][row] = bad
    cap = 4 * sum(r["n_rows"] for r in recs)
    _expect(H.GpuUnpack(ctx, recs, cap), toks, dropped, B.MW_FLAG_BAD_SRC_TOKEN, cap)
    ctx.close()


def test_row_without_a_local_expert_and_ids_out_of_range():
    ctx = H.make_ctx(W_SMALL, MY_RANK)
    recs, toks = _regions(ctx)
    e2r = W.expert_to_rank(W_SMALL)
    elsewhere = int(np.nonzero(e2r != MY_RANK)[0][0])
    t = int(H.host(recs[2]["row_src_token"])[1])
    recs[2]["row_topk"][1] = torch.tensor([elsewhere, -1], dtype=torch.int32)     # addressed, but to no expert here
    cap = 4 * sum(r["n_rows"] for r in recs)
    _expect(H.GpuUnpack(ctx, recs, cap), toks, [(2, t)], B.MW_FLAG_NO_LOCAL_EXPERT, cap)
    # an id outside [0, E): ignored and flagged; the row keeps its other expert
    recs2, toks2 = _regions(ctx)
    row_tk = H.host(recs2[5]["row_topk"])[0].copy()
    keep = [int(e) for e in row_tk if e >= 0 and e2r[e] == MY_RANK]
    recs2[5]["row_topk"][0] = torch.tensor([keep[0], W_SMALL.n_experts + 7], dtype=torch.int32)
    t5 = int(H.host(recs2[5]["row_src_token"])[0])
    fixed = [(tk.copy(), x, sc) for tk, x, sc in toks2]
    fixed[5][0][t5] = np.array([keep[0], -1], dtype=np.int32)
    gu = H.GpuUnpack(ctx, recs2, cap)
    assert int(gu.stats["error_flags"]) == B.MW_FLAG_BAD_EXPERT
    want = ref.dispatch_plain(fixed, e2r, MY_RANK, cap)
    o = gu.host_out()
    H.assert_same_bytes(o[3], want[3], "out_src_token")
    H.assert_same_bytes(o[0], want[0], "out_rows")
    ctx.close()


def test_descriptor_beyond_the_region_is_dropped():
    ctx = H.make_ctx(W_SMALL, MY_RANK)
    recs, toks = _regions(ctx)
    d = H.host(recs[6]["desc"]).reshape(-1).view(B.DESC_DTYPE).copy()
    g = recs[6]["n_desc"] - 1
    off, cnt = int(d["row_offset"][g]), int(d["row_count"][g])
    dropped = [(6, int(t)) for t in H.host(recs[6]["row_src_token"])[off:off + cnt]]
    d["row_count"][g] = cnt + 1000
    recs[6]["desc"] = H.dev(d.view(np.uint8).reshape(-1, B.DESC_BYTES))
    cap = 4 * sum(r["n_rows"] for r in recs)
    _expect(H.GpuUnpack(ctx, recs, cap), toks, dropped, B.MW_FLAG_BAD_DESC, cap)
    ctx.close()


def test_duplicate_source_token_is_flagged():
    ctx = H.make_ctx(W_SMALL, MY_RANK)
    recs, toks = _regions(ctx)
    src = H.host(recs[0]["row_src_token"])
    rtk = H.host(recs[0]["row_topk"])
    e2r = W.expert_to_rank(W_SMALL)
    local = lambda row: {int(e) for e in rtk[row] if e >= 0 and e2r[e] == MY_RANK}
    pair = next((a, b) for a in range(len(src)) for b in range(a + 1, len(src)) if local(a) & local(b))
    recs[0]["row_src_token"][pair[1]] = int(src[pair[0]])
    cap = 4 * sum(r["n_rows"] for r in recs)
    gu = H.GpuUnpack(ctx, recs, cap)                       # what is delivered for the pair is unspecified
    assert int(gu.stats["error_flags"]) == B.MW_FLAG_DUP_SRC_TOKEN
    # the flag does not stick and the context still works
    recs2, toks2 = _regions(ctx)
    _expect(H.GpuUnpack(ctx, recs2, cap), toks2, [], 0, cap)
    ctx.close()


def test_more_rows_than_the_context_was_created_for():
    w = W_SMALL
    full, _ = _regions(H.make_ctx(w, MY_RANK))
    total = sum(r["n_rows"] for r in full)
    keep_rows = total // 2
    ctx = H.make_ctx(w, MY_RANK, max_recv_rows=keep_rows)
    recs, toks = _regions(ctx)
    dropped, seen, flag = [], 0, B.MW_FLAG_RECV_CAPACITY
    for p, r in enumerate(recs):                            # regions are taken in peer order until the rows run out
        src = H.host(r["row_src_token"])[: r["n_rows"]]
        kept_n = max(0, min(r["n_rows"], keep_rows - seen))
        if kept_n < r["n_rows"]:
            # a group that reaches beyond the rows taken is dropped as a whole (its descriptor no
            # longer fits the region) and flagged as such
            d = H.host(r["desc"]).reshape(-1).view(B.DESC_DTYPE)[: r["n_desc"]]
            for g in range(r["n_desc"]):
                off, cnt = int(d["row_offset"][g]), int(d["row_count"][g])
                if off + cnt > kept_n:
                    dropped += [(p, int(t)) for t in src[off:off + cnt]]
                    flag |= B.MW_FLAG_BAD_DESC
        seen += r["n_rows"]
    cap = 4 * total
    gu = H.GpuUnpack(ctx, recs, cap)
    assert int(gu.stats["n_rows_seen"]) == keep_rows
    _expect(gu, toks, dropped, flag, cap)
    ctx.close()
    # a peer that claims more rows than max_tokens: its surplus rows are not looked at
    ctx = H.make_ctx(w, MY_RANK, max_tokens=8)
    recs, toks = _regions(H.make_ctx(w, MY_RANK))
    dropped = []
    for p, r in enumerate(recs):
        src = H.host(r["row_src_token"])[: r["n_rows"]]
        dropped += [(p, int(t)) for i, t in enumerate(src) if i >= 8 or t >= 8]
    gu = H.GpuUnpack(ctx, recs, cap)
    assert int(gu.stats["error_flags"]) & B.MW_FLAG_RECV_CAPACITY
    assert int(gu.stats["n_rows_seen"]) == sum(min(r["n_rows"], 8) for r in recs)
    ctx.close()


def _ride_setup(w, n_peers, peer_tokens, my_rank=1):
    """Two contexts, a small received batch indexed in the first, buffers for a plan in the second."""
    ctxs = [H.make_ctx(w, my_rank, max_recv_rows=n_peers * peer_tokens), H.make_ctx(w, my_rank, max_recv_rows=n_peers * peer_tokens)]
    recs, toks = [], []
    for p in range(n_peers):
        tk = W.topk_ids(w, 1, p)[:peer_tokens]
        x, _ = W.payload_rows(w, 1, p, np.arange(peer_tokens))
        recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, None).deliver(my_rank)))
        toks.append((tk, x, None))
    cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
    table = B.peers_table(recs, H.DEV)
    bufs = [B.RecvBuffers(ctxs[0], cap), B.RecvBuffers(ctxs[1], cap)]
    return ctxs, toks, cap, (table, recs), bufs      # (the table points into recs: both stay alive)


def _ride(ctxs, w, n_peers, cap, table, bufs, tk_d, sb):
    """Expander of ctxs[0]'s batch with the index and the plan of `tk_d` riding into ctxs[1]."""
    table = table[0]
    ctxs[0].mw_unpack_index(table, n_peers, cap, bufs[0].expert_offsets, bufs[0].stats)
    ctxs[0].mw_unpack_expand_index_plan_next(n_peers, bufs[0].out_rows, None, cap, bufs[0].out_src_peer,
                                             bufs[0].out_src_token, ctxs[1], table, n_peers, cap,
                                             bufs[1].expert_offsets, bufs[1].stats, tk_d, sb.mask, sb.perm,
                                             sb.desc, sb.stats)
    torch.cuda.synchronize()
    return ctxs[1].mw_get_send_stats(sb.stats)


def _check_plan(w, sb, st, tk):
    m, perm, desc, ost = ref.plan(tk, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    assert int(st["error_flags"]) == 0
    for f in ("n_rows", "n_groups", "multicast_bytes", "unicast_bytes"):
        assert int(st[f]) == int(ost[f]), f
    H.assert_same_bytes(st["rows_per_dest"], ost["rows_per_dest"], "rows_per_dest")
    H.assert_same_bytes(H.host(sb.mask).view(np.uint64)[: len(tk)], m, "mask")
    H.assert_same_bytes(H.host(sb.perm)[: len(perm)], perm, "perm")
    H.assert_same_bytes(H.host(sb.desc).reshape(-1).view(B.DESC_DTYPE)[: len(desc)].view(np.uint8), desc.view(np.uint8), "desc")


def test_riding_plan_gives_up_and_the_context_plans_again():
    """mw_ctx_set_ride_wait_limit(0): the second half of a riding plan looks once and does not
    wait.  The first half is made long by construction -- 8192 tokens over 256 ranks, a thousand
    ranking workgroups of several memory round trips each, dispatched a fraction of a
    microsecond before the finishing ones -- so the plan MUST be given up: the statistics say
    MW_FLAG_PLAN_TIMEOUT with zero rows, every kernel ends normally, the receive side of the same
    launch is exact.  The context is not lost: the launch leaves its plan state clean, and the
    next plans on it -- mw_plan, then a riding plan with the default limit -- are the oracle's."""
    w = W.DispatchWorkload("giveup", 41, 256, 256, 8, 8192, 256, "bf16", "uniform")
    n_peers, peer_tokens = 6, 300
    ctxs, toks, cap, table, bufs = _ride_setup(w, n_peers, peer_tokens)
    sb = B.SendBuffers(ctxs[1], w.n_tokens)
    tk_me = W.topk_ids(w, 2, 1)
    tk_d = H.dev(tk_me)
    ctxs[1].mw_ctx_set_ride_wait_limit(0)
    st = _ride(ctxs, w, n_peers, cap, table, bufs, tk_d, sb)
    assert int(st["error_flags"]) == B.MW_FLAG_PLAN_TIMEOUT
    assert (int(st["n_rows"]), int(st["n_groups"]), int(st["multicast_bytes"]), int(st["unicast_bytes"])) == (0, 0, 0, 0)
    assert not st["rows_per_dest"].any()
    e2r = W.expert_to_rank(w)
    want = ref.dispatch_plain(toks, e2r, 1, cap)
    for c, b in zip(ctxs, bufs):                          # the expander of the launch and its riding index
        if c is ctxs[1]:
            c.mw_unpack_expand(n_peers, b.out_rows, None, cap, b.out_src_peer, b.out_src_token)
        rs = c.mw_get_recv_stats(b.stats)
        q = int(rs["n_out_rows"])
        assert int(rs["error_flags"]) == 0 and q == len(want[2])
        H.assert_same_bytes(H.host(b.out_rows)[:q], want[0], "out_rows beside a plan that gave up")
        H.assert_same_bytes(H.host(b.out_src_token)[:q], want[3], "out_src_token beside a plan that gave up")
    # the same context plans again: call by call ...
    ctxs[1].mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
    _check_plan(w, sb, ctxs[1].mw_get_send_stats(sb.stats), tk_me)
    # ... gives up once more, with another batch (nothing of the first attempt may linger) ...
    tk2 = W.topk_ids(w, 3, 1)[:5000]
    st = _ride(ctxs, w, n_peers, cap, table, bufs, H.dev(tk2), sb)
    assert int(st["error_flags"]) == B.MW_FLAG_PLAN_TIMEOUT and int(st["n_rows"]) == 0
    # ... and rides with the default limit
    ctxs[1].mw_ctx_set_ride_wait_limit(1 << 21)
    sb2 = B.SendBuffers(ctxs[1], w.n_tokens)
    st = _ride(ctxs, w, n_peers, cap, table, bufs, tk_d, sb2)
    _check_plan(w, sb2, st, tk_me)
    with pytest.raises(B.MwError):
        ctxs[1].mw_ctx_set_ride_wait_limit(-1)
    for c in ctxs:
        c.close()


def test_riding_plan_with_the_default_limit_is_the_oracles():
    """The same launch with the default wait limit, batch after batch on one pair of contexts
    (sizes going down and up again, so a finishing workgroup count that changes from launch to
    launch finds clean state): every plan complete and exact, never a time-out flag."""
    w = W.DispatchWorkload("ride", 42, 64, 256, 8, 4096, 256, "bf16", "uniform")
    n_peers, peer_tokens = 5, 200
    ctxs, toks, cap, table, bufs = _ride_setup(w, n_peers, peer_tokens)
    for i, n in enumerate((4096, 700, 1, 0, 2049)):
        tk = W.topk_ids(w, 10 + i, 1)[:n]
        sb = B.SendBuffers(ctxs[1], max(n, 1))
        st = _ride(ctxs, w, n_peers, cap, table, bufs, H.dev(tk) if n else torch.zeros((0, w.top_k), dtype=torch.int32, device=H.DEV), sb)
        _check_plan(w, sb, st, tk)
    for c in ctxs:
        c.close()
