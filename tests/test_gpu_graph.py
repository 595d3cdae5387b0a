"""GPU: the entry points only enqueue kernels and keep no state on the host between calls, so a
step can be captured into a HIP graph (through torch's capture of the current stream) and
replayed.  Every replay is checked against the CPU oracle, with the program's own eager work --
other plans on the same context, cleared outputs, fresh inputs -- and synchronisations between
the replays."""
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


def _clear(*tensors):
    for t in tensors:
        if t is not None:
            t.zero_()


def _check_send_buffers(w, sb, ctx, tk, x, sc):
    e2r = W.expert_to_rank(w)
    m, perm, desc, ost = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    packed, src, rtk = ref.pack(x, sc, tk, perm)
    st = ctx.mw_get_send_stats(sb.stats)
    N, G = int(st["n_rows"]), int(st["n_groups"])
    assert (N, G, int(st["error_flags"])) == (len(perm), len(desc), 0)
    H.assert_same_bytes(H.host(sb.mask).view(np.uint64)[: len(tk)], m, "mask")
    H.assert_same_bytes(H.host(sb.perm)[:N], perm, "perm")
    H.assert_same_bytes(H.host(sb.desc).reshape(-1).view(B.DESC_DTYPE)[:G].view(np.uint8), desc.view(np.uint8), "desc")
    H.assert_same_bytes(st["rows_per_dest"], ost["rows_per_dest"], "rows_per_dest")
    assert int(st["unicast_bytes"]) == int(ost["unicast_bytes"])
    H.assert_same_bytes(H.host(sb.packed)[:N], packed, "packed rows")
    H.assert_same_bytes(H.host(sb.row_src_token)[:N], src, "row_src_token")
    H.assert_same_bytes(H.host(sb.row_topk)[:N], rtk, "row_topk")


@pytest.mark.parametrize("fused", [False, True])
def test_captured_step_replays(fused):
    """plan + pack (or the one-launch mw_plan_pack) and unpack of received regions in one graph;
    four replays, the sender's inputs replaced before each, eager plans of other batch sizes on
    the same context in between."""
    T = 200 if fused else 333
    w = W.DispatchWorkload("graph", 77, 8, 16, 2, T, 256, "bf16", "uniform")
    my_rank, e2r = 3, W.expert_to_rank(w)
    _say("graph replay", "fused" if fused else "plan+pack", "T", T)
    ctx = H.make_ctx(w, my_rank, max_tokens=512)

    # what this rank receives: every peer's delivery, built eagerly once (GPU) / by the oracle
    recs, bufs = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, 1, p)
        x, sc = W.payload_rows(w, 1, p)
        recs.append(H.shrink(H.GpuSend(ctx, tk, x, sc).deliver(my_rank)))
        _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        packed, src, rtk = ref.pack(x, sc, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
    cap = max(1, sum(r["n_rows"] for r in recs) * 2)
    expect_recv = ref.unpack(bufs, w.top_k, e2r, my_rank, 2 * w.hidden, 0, cap)
    table = B.peers_table(recs, H.DEV)

    # the graph's fixed buffers
    tk_d = torch.zeros((T, w.top_k), dtype=torch.int32, device=H.DEV)
    x_d = torch.zeros((T, w.hidden), dtype=torch.int16, device=H.DEV)
    sb, rv = B.SendBuffers(ctx, T), B.RecvBuffers(ctx, cap)
    other = B.SendBuffers(ctx, 512)

    def step():
        if fused:
            ctx.mw_plan_pack(tk_d, x_d, None, sb.mask, sb.perm, sb.desc, sb.stats, sb.packed, sb.row_src_token,
                             sb.row_topk)
        else:
            ctx.mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
            ctx.mw_pack(x_d, None, tk_d, sb.perm, sb.stats, sb.packed, sb.row_src_token, sb.row_topk)
        ctx.mw_unpack(table, w.n_ranks, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token,
                      rv.expert_offsets, rv.stats)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                            # once eagerly on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    class _Got:                                           # what check_unpack reads
        pass

    for rep in range(4):
        seed = 10 + rep
        tk = W.topk_ids(w, seed, my_rank)
        if rep == 2:
            tk[::7] = -1                                  # fewer rows than the capture saw
        x, _ = W.payload_rows(w, seed, my_rank)
        tk_d.copy_(H.dev(tk))
        x_d.copy_(H.dev(x).view(torch.int16))
        # eager work on the same context between the replays: plans of other sizes
        for t_other in (512, 57):
            ow = W.scaled(w, n_tokens=t_other)
            ctx.mw_plan(H.dev(W.topk_ids(ow, seed, 0)), other.mask, other.perm, other.desc, other.stats)
        _clear(sb.mask, sb.desc, sb.stats, sb.packed, sb.row_topk, rv.out_rows, rv.expert_offsets, rv.stats)
        sb.perm.fill_(-1); sb.row_src_token.fill_(-1); rv.out_src_peer.fill_(-1); rv.out_src_token.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _say("  replay", rep)
        _check_send_buffers(w, sb, ctx, tk, x, None)
        g = _Got()
        g.ctx, g.buf = ctx, rv
        g.stats = ctx.mw_get_recv_stats(rv.stats)
        g.Q = int(g.stats["n_out_rows"])
        g.host_out = lambda: H.GpuUnpack.host_out(g)
        H.check_unpack(g, expect_recv, "replay %d" % rep)
        # and the eager calls still agree after a replay
        if rep == 1:
            step()
            torch.cuda.synchronize()
            _check_send_buffers(w, sb, ctx, tk, x, None)
    ctx.close()


def test_captured_allgather_step_replays():
    """mw_allgather_step in a graph: three replays, the shard to send and the shards received
    replaced before each, an eager AllGather plan of another size on the same context in between."""
    w = W.AllGatherWorkload("ag_graph", 43, 8, 3000 * 8)
    _say("graph replay allgather step", w.shard_bytes)
    ctx = B.Context(w.n_ranks, 0, 1, w.my_rank, 0, B.MW_ROW_BYTES, 1, 0, None, row_bytes=w.shard_bytes,
                    device=H.DEV)
    own = torch.zeros(w.shard_elems, dtype=torch.int16, device=H.DEV)
    send = torch.zeros_like(own)
    recv = [torch.zeros_like(own) for _ in range(w.n_ranks)]
    table = torch.tensor([t.data_ptr() for t in recv], dtype=torch.int64, device=H.DEV)
    out = torch.zeros(w.n_ranks * w.shard_elems, dtype=torch.int16, device=H.DEV)
    desc = torch.zeros(B.DESC_BYTES, dtype=torch.uint8, device=H.DEV)
    stats = torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    d2, s2 = torch.zeros_like(desc), torch.zeros_like(stats)

    def step():
        ctx.mw_allgather_step(own, w.shard_bytes, send, desc, stats, table, out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    od, ost = ref.plan_allgather(w.n_ranks, w.shard_bytes)
    for rep in range(3):
        shards = [W.allgather_shard(w, 20 + rep, r) for r in range(w.n_ranks)]
        mine = W.allgather_shard(w, 30 + rep, w.my_rank)
        for t, a in zip(recv, shards):
            t.copy_(H.dev(a).view(torch.int16))
        own.copy_(H.dev(mine).view(torch.int16))
        ctx.mw_plan_allgather(4096, d2, s2)
        _clear(send, out, desc, stats)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _say("  replay", rep)
        H.assert_same_bytes(H.host(out).view(np.uint8), ref.unpack_allgather(shards), "replay: gathered output")
        H.assert_same_bytes(H.host(send), ref.pack_allgather(mine).view(np.uint16), "replay: send buffer")
        H.assert_same_bytes(H.host(desc), od.view(np.uint8).reshape(-1), "replay: desc")
        H.assert_same_bytes(np.array([ctx.mw_get_send_stats(stats)]).view(np.uint8),
                            np.array([ost]).view(np.uint8), "replay: stats")
    ctx.close()


def test_captured_stream_step_replays():
    """mw_stream_step (pack, expand, the next batch's index and plan in one launch, with its
    workgroups that wait for others of the same launch) in a graph: three replays with new tokens,
    payload and received regions each time, the eager calls a stream needs around it in between
    (plan of the batch it packs, index of the batch it expands, expander of the batch it indexed)."""
    w = W.scaled(W.C1, n_tokens=200, hidden=512)
    my_rank, e2r, T, R = 5, W.expert_to_rank(w), 200, W.C1.n_ranks
    _say("graph replay stream step")
    ctxs = [H.make_ctx(w, my_rank), H.make_ctx(w, my_rank)]
    # two sets of received regions (device buffers stay, the graph's record table is overwritten)
    sets = []
    for seed in (1, 2):
        recs, toks = [], []
        for p in range(R):
            tk = W.topk_ids(w, seed, p)
            x, sc = W.payload_rows(w, seed, p)
            recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, sc).deliver(my_rank)))
            toks.append((tk, x, sc))
        sets.append(dict(recs=recs, toks=toks, table=B.peers_table(recs, H.DEV)))
    cap = max(sum(r["n_rows"] for r in s["recs"]) for s in sets) * 2
    want = [ref.dispatch_plain(s["toks"], e2r, my_rank, cap) for s in sets]
    cur_table, next_table = torch.zeros_like(sets[0]["table"]), torch.zeros_like(sets[0]["table"])
    tk_d = torch.zeros((T, w.top_k), dtype=torch.int32, device=H.DEV)        # batch that is packed
    x_d = torch.zeros((T, w.hidden), dtype=torch.int16, device=H.DEV)
    tkn_d = torch.zeros((T, w.top_k), dtype=torch.int32, device=H.DEV)       # batch that is planned
    sb, sn = B.SendBuffers(ctxs[0], T), B.SendBuffers(ctxs[1], T)
    rv, rvn = B.RecvBuffers(ctxs[0], cap), B.RecvBuffers(ctxs[1], cap)

    def step():
        ctxs[0].mw_stream_step(x_d, None, tk_d, sb.perm, sb.stats, sb.packed, sb.row_src_token, sb.row_topk, R,
                               rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token, ctxs[1], next_table,
                               R, cap, rvn.expert_offsets, rvn.stats, tkn_d, sn.mask, sn.perm, sn.desc, sn.stats)

    def eager_before(rep):
        """What a stream has done before this step: inputs in place, this batch planned and indexed."""
        tk, tkn = W.topk_ids(w, 40 + rep, my_rank), W.topk_ids(w, 50 + rep, my_rank)
        if rep == 1:
            tkn[::4] = -1
        x, _ = W.payload_rows(w, 40 + rep, my_rank)
        tk_d.copy_(H.dev(tk)); tkn_d.copy_(H.dev(tkn)); x_d.copy_(H.dev(x).view(torch.int16))
        cur_table.copy_(sets[rep % 2]["table"]); next_table.copy_(sets[(rep + 1) % 2]["table"])
        _clear(sb.packed, sb.row_topk, sn.mask, sn.desc, sn.stats, rv.out_rows, rvn.expert_offsets, rvn.stats)
        sb.row_src_token.fill_(-1); sn.perm.fill_(-1); rv.out_src_peer.fill_(-1); rv.out_src_token.fill_(-1)
        ctxs[0].mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
        ctxs[0].mw_unpack_index(cur_table, R, cap, rv.expert_offsets, rv.stats)
        torch.cuda.synchronize()
        return tk, tkn, x

    side = torch.cuda.Stream()
    eager_before(0)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager_before(0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    class _Got:
        pass

    for rep in range(3):
        tk, tkn, x = eager_before(rep)
        graph.replay()
        torch.cuda.synchronize()
        _say("  replay", rep)
        # packed: batch tk
        _check_send_buffers(w, sb, ctxs[0], tk, x, None)
        # planned: batch tkn
        m, perm, desc, ost = ref.plan(tkn, e2r, R, w.row_bytes)
        st = ctxs[1].mw_get_send_stats(sn.stats)
        n, g_ = int(st["n_rows"]), int(st["n_groups"])
        assert (n, g_, int(st["error_flags"])) == (len(perm), len(desc), 0)
        H.assert_same_bytes(H.host(sn.mask).view(np.uint64)[:T], m, "replay: next mask")
        H.assert_same_bytes(H.host(sn.perm)[:n], perm, "replay: next perm")
        H.assert_same_bytes(H.host(sn.desc).reshape(-1).view(B.DESC_DTYPE)[:g_].view(np.uint8), desc.view(np.uint8),
                            "replay: next desc")
        # expanded: the set indexed eagerly; indexed: the other set, expanded eagerly now
        ctxs[1].mw_unpack_expand(R, rvn.out_rows, rvn.out_scales, cap, rvn.out_src_peer, rvn.out_src_token)
        torch.cuda.synchronize()
        for c_, b_, wnt, what in ((ctxs[0], rv, want[rep % 2], "expanded"), (ctxs[1], rvn, want[(rep + 1) % 2], "indexed")):
            g = _Got()
            g.ctx, g.buf = c_, b_
            g.stats = c_.mw_get_recv_stats(b_.stats)
            g.Q = int(g.stats["n_out_rows"])
            g.host_out = lambda g=g: H.GpuUnpack.host_out(g)
            H.check_unpack(g, wnt, "replay %d %s" % (rep, what))
    for c in ctxs:
        c.close()
