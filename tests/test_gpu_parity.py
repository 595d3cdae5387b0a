"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Bar: bit-exact on every index, descriptor, statistic and payload
byte (the path is pure data movement and integer work; nothing is rounded)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_22428_amd import binding as B
from paper_2605_22428_amd import workloads as W

import gpu_harness as H

pytestmark = pytest.mark.gpu

SEEDS = [W.BASE_SEED, 1, 2]


def _say(*a):
    print(*a, flush=True)


def run_dispatch(w, seed, my_rank, check_all_senders=True, lazy=False, tier2=True, also_full=False,
                 sample_peers=(), stream_step=False, row_stride=0):
    """Every simulated peer runs plan+pack (GPU and oracle separately), the simulated network
    filters to my_rank, then unpack on both sides; compared at every stage."""
    _say("dispatch", w.name, "seed", seed, "my_rank", my_rank, "T", w.n_tokens, "H", w.hidden)
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, my_rank, row_stride=row_stride)
    recs, full_recs, bufs, toks = [], [], [], []
    topks = W.topk_ids_many(w, seed, range(w.n_ranks))
    x_dev = s_dev = None
    if lazy:
        xdt = torch.uint8 if w.row_format == "fp8" else torch.int16
        x_dev = torch.zeros((w.n_tokens, w.hidden), dtype=xdt, device=H.DEV)
        if w.row_format == "fp8":
            s_dev = torch.zeros((w.n_tokens, w.hidden // 128), dtype=torch.float32, device=H.DEV)
    for p in range(w.n_ranks):
        tk = topks[p]
        detailed = check_all_senders or p == my_rank or p in sample_peers
        pre = 0xA5 if detailed else 0
        tokens = None
        if lazy and not detailed:
            # only the rows addressed to my_rank are drawn (the others are zero on both sides);
            # the generator's choice of rows is checked against what is delivered further down
            tokens = W.tokens_for_rank(w, tk, my_rank)
            rows, sc_rows = W.payload_rows(w, seed, p, tokens)
            x = np.zeros((w.n_tokens, w.hidden), dtype=rows.dtype)
            x[tokens] = rows
            sc = None
            idx = torch.from_numpy(tokens).to(H.DEV)
            x_dev.zero_()
            x_dev[idx] = H.dev(rows).view(x_dev.dtype)
            if sc_rows is not None:
                sc = np.zeros((w.n_tokens, w.hidden // 128), dtype=np.float32)
                sc[tokens] = sc_rows
                s_dev.zero_()
                s_dev[idx] = H.dev(sc_rows)
            g = H.GpuSend(ctx, tk, x, sc, x_dev=x_dev, scales_dev=s_dev)
        else:
            # this rank's own batch and the sampled peers: every row drawn, every packed row compared
            x, sc = W.payload_rows(w, seed, p)
            g = H.GpuSend(ctx, tk, x, sc, prefill=pre)
        toks.append((tk, x, sc))
        if detailed or tier2:
            if detailed:
                perm, desc, packed, src, rtk = H.check_send(w, g, tk, x, sc)
            else:
                _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
                packed, src, rtk = ref.pack(x, sc, tk, perm)
            obuf = ref.deliver(desc, packed, src, rtk, my_rank)
            bufs.append(obuf)
        rec = H.shrink(g.deliver(my_rank))
        if tokens is not None:
            assert rec["n_rows"] == len(tokens), "payload was drawn for other rows than those delivered"
        if detailed:
            got = H.record_host(rec, w.row_bytes)
            for a, b, name in zip(got, obuf, ("desc", "rows", "src_token", "row_topk")):
                H.assert_same_bytes(a.view(np.uint8) if name == "desc" else a,
                                    b.view(np.uint8) if name == "desc" else b, "deliver %s peer %d" % (name, p))
        recs.append(rec)
        if also_full:
            fr = g.full_record()
            full_recs.append(dict(desc=fr["desc"].clone(), rows=fr["rows"].clone(),
                                  row_src_token=fr["row_src_token"].clone(), row_topk=fr["row_topk"].clone(),
                                  n_desc=fr["n_desc"], n_rows=fr["n_rows"]))
        del g
    xrb = 2 * w.hidden if w.row_format == "bf16" else w.hidden
    srb = w.row_bytes - xrb
    m_rows = sum(r["n_rows"] for r in recs)
    cap = max(1, m_rows * min(w.top_k, w.experts_per_rank))
    o1 = ref.dispatch_plain(toks, e2r, my_rank, cap)
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, o1, "vs plain definition")
    assert int(gu.stats["n_recv_rows"]) == m_rows
    if tier2:
        o2 = ref.unpack(bufs, w.top_k, e2r, my_rank, xrb, srb, cap)
        H.check_unpack(gu, o2, "vs oracle unpack")
    if also_full:
        gf = H.GpuUnpack(ctx, full_recs, cap)
        H.check_unpack(gf, o1, "complete sender buffers")
    if stream_step:
        # the same batch through mw_stream_step, the launch bench.py times by default: this rank's
        # own tokens are packed, the received regions expanded, and the same regions / the same
        # tokens indexed and planned again as "the next batch" in a second context
        tk, x, sc = toks[my_rank]
        g = H.GpuSend(ctx, tk, x, sc)                          # (plans; its packed rows are overwritten below)
        ctx2 = H.make_ctx(w, my_rank, row_stride=row_stride)
        rv, rv2 = B.RecvBuffers(ctx, cap), B.RecvBuffers(ctx2, cap)
        nxt = B.SendBuffers(ctx2, w.n_tokens)
        table = B.peers_table(recs, H.DEV)
        ctx.mw_unpack_index(table, len(recs), cap, rv.expert_offsets, rv.stats)
        g.buf.packed.zero_(); g.buf.row_src_token.fill_(-1); g.buf.row_topk.zero_()
        ctx.mw_stream_step(g.x_d, g.s_d, g.topk_d, g.buf.perm, g.buf.stats, g.buf.packed, g.buf.row_src_token,
                           g.buf.row_topk, len(recs), rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                           rv.out_src_token, ctx2, table, len(recs), cap, rv2.expert_offsets, rv2.stats, g.topk_d,
                           nxt.mask, nxt.perm, nxt.desc, nxt.stats)
        ctx2.mw_unpack_expand(len(recs), rv2.out_rows, rv2.out_scales, cap, rv2.out_src_peer, rv2.out_src_token)
        torch.cuda.synchronize()
        H.check_send(w, g, tk, x, sc)                          # plan of before, rows packed by the step
        for c_, b_, what in ((ctx, rv, "stream step: expanded"), (ctx2, rv2, "stream step: indexed for the next")):
            gs = H.GpuUnpack.__new__(H.GpuUnpack)
            gs.ctx, gs.buf = c_, b_
            gs.stats = c_.mw_get_recv_stats(b_.stats)
            gs.Q = int(gs.stats["n_out_rows"])
            H.check_unpack(gs, o1, what)
        g2 = H.GpuSend.__new__(H.GpuSend)                      # the plan the step made, in GpuSend's clothes
        g2.ctx, g2.T, g2.buf = ctx2, w.n_tokens, nxt
        g2.stats = ctx2.mw_get_send_stats(nxt.stats)
        g2.N, g2.G = int(g2.stats["n_rows"]), int(g2.stats["n_groups"])
        m_, perm_, desc_, st_ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        gm, gperm, gdesc = g2.host_plan()
        H.assert_same_bytes(gm, m_, "stream step: next mask")
        H.assert_same_bytes(gperm, perm_, "stream step: next perm")
        H.assert_same_bytes(gdesc.view(np.uint8), desc_.view(np.uint8), "stream step: next desc")
        assert int(g2.stats["unicast_bytes"]) == int(st_["unicast_bytes"]) and int(g2.stats["error_flags"]) == 0
        ctx2.close()
    _say("  rows received", m_rows, "output rows", gu.Q)
    ctx.close()
    return gu


# ------------------------------------------------------------------ configs at oracle-friendly sizes
@pytest.mark.parametrize("seed", SEEDS)
@pytest.mark.parametrize("my_rank", [0, 5])
def test_c0_tiny(seed, my_rank):
    run_dispatch(W.C0, seed, my_rank, also_full=True, stream_step=True)


@pytest.mark.parametrize("seed", SEEDS)
def test_c1_shape_reduced(seed):
    # 64 ranks, 256 experts, top-8, group-limited routing; 333 tokens (ragged), 1024-wide rows
    run_dispatch(W.scaled(W.C1, n_tokens=333, hidden=1024), seed, 37, also_full=(seed == 1), stream_step=True)


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_c2_shape_reduced_fp8(seed):
    run_dispatch(W.scaled(W.C2, n_tokens=333, hidden=1024), seed, 0, also_full=(seed == 1), stream_step=True)


@pytest.mark.parametrize("which", ["median", "hottest"])
def test_c3_shape_reduced(which):
    w = W.scaled(W.C3, n_tokens=200, hidden=512)
    r = W.zipf_median_rank(w, 1) if which == "median" else W.zipf_hottest_rank(w, 1)
    run_dispatch(w, 1, r, check_all_senders=False, sample_peers=(0, 100, 255))


def test_wide_rows_ragged_tail():
    # full-width bf16 and fp8 rows, token count not a multiple of any tile
    run_dispatch(W.DispatchWorkload("wide_bf16", 11, 8, 16, 2, 257, 7168, "bf16", "uniform"), 1, 3)
    run_dispatch(W.DispatchWorkload("wide_fp8", 12, 8, 16, 2, 129, 7168, "fp8", "uniform"), 1, 6)


# ------------------------------------------------------------------ full sizes
def test_c1_full_size():
    run_dispatch(W.C1, W.BASE_SEED, 0, check_all_senders=False, lazy=True, sample_peers=(7, 63), stream_step=True)


def test_c2_full_size_fp8():
    run_dispatch(W.C2, W.BASE_SEED, 0, check_all_senders=False, lazy=True, tier2=False, sample_peers=(31,),
                 stream_step=True)


def test_c3_full_size_send_side():
    w = W.C3
    tk = W.topk_ids(w, W.BASE_SEED, 0)
    tokens = np.arange(0, w.n_tokens, 7)
    x, _ = W.payload_full(w, W.BASE_SEED, 0, tokens)
    ctx = H.make_ctx(w, 0, max_recv_rows=1)
    g = H.GpuSend(ctx, tk, x, None)
    H.check_send(w, g, tk, x, None)
    assert int(g.stats["unicast_bytes"]) == 8 * int(g.stats["multicast_bytes"])
    ctx.close()


def test_c3_full_size_receive_median_rank():
    w = W.C3
    r = W.zipf_median_rank(w, W.BASE_SEED)
    run_dispatch(W.scaled(w, my_rank=r), W.BASE_SEED, r, check_all_senders=False, lazy=True, tier2=False,
                 sample_peers=(0, 255))


def _pooled_regions(w, seed, my_rank, ctx, sample_peers):
    """Every peer's plan + pack + delivery to my_rank with pooled payload (every row drawn, no two
    equal); the sampled peers' send side is compared with the oracle row by row."""
    recs, toks = [], []
    for p, tk in enumerate(W.topk_ids_many(w, seed, range(w.n_ranks))):
        x = W.payload_rows_pooled(w, seed, p)
        g = H.GpuSend(ctx, tk, x, None, prefill=0x5A if p in sample_peers else 0)
        if p in sample_peers:
            H.check_send(w, g, tk, x, None)
        recs.append(H.shrink(g.deliver(my_rank)))
        toks.append((tk, x, None))
        del g
    return recs, toks


def test_c3_hottest_rank_512_tokens_per_peer_full_rows():
    """The skew stress point of the large-EP configuration: the rank of the most popular expert
    receives from 256 peers of 512 tokens each, rows of the full 14336 bytes -- more than a
    hundred thousand rows (1.6 GB), one peer's region after the other nearly full, several times
    more rows than the expander's grid has workgroup rows.  Whole output against the plain
    definition."""
    w = W.scaled(W.C3, n_tokens=512)
    r = W.zipf_hottest_rank(w, W.BASE_SEED)
    ctx = H.make_ctx(w, r)
    recs, toks = _pooled_regions(w, W.BASE_SEED, r, ctx, sample_peers=(r, 17))
    m_rows = sum(rec["n_rows"] for rec in recs)
    _say("hottest rank", r, "rows received", m_rows)
    assert m_rows > 3 * 32768                                  # (the point of the case)
    cap = m_rows
    want = ref.dispatch_plain(toks, W.expert_to_rank(w), r, cap)
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, want, "hottest rank vs plain definition")
    assert int(gu.stats["n_recv_rows"]) == m_rows == gu.Q
    ctx.close()


@pytest.mark.parametrize("schedule", ["launch_and_plan", "one_launch"])
def test_stream_of_full_size_steps_as_the_bench_issues_them(schedule):
    """The two schedules bench.py times, issued exactly as it issues them, for four steps in a row
    without a synchronisation in between, at full size.  "launch_and_plan" (the large-EP
    configuration, 8192 tokens over 256 ranks): mw_stream_step with an EMPTY batch to plan (NULL plan
    outputs, a statistics block nobody reads) packs batch n, expands received batch n and indexes
    received batch n + 1, while mw_plan of batch n + 1 runs on a third context on a second stream,
    one event each way.  "one_launch" (the DeepSeek-V3-shaped configuration): the plan of batch
    n + 1 rides in the launch.  Every batch this rank sends is different; everything each step
    wrote is compared with the oracle afterwards."""
    if schedule == "launch_and_plan":
        w0 = W.C3
        my_rank = W.zipf_median_rank(w0, W.BASE_SEED)
        peer_tokens = 1024        # per peer on the receive side: 256 full regions would be minutes of oracle time
    else:
        w0, my_rank, peer_tokens = W.C1, 0, 1024
    w = W.scaled(w0, my_rank=my_rank)
    wr = W.scaled(w, n_tokens=peer_tokens)
    e2r = W.expert_to_rank(w)
    R, K, T = w.n_ranks, w.top_k, w.n_tokens
    rctx = [H.make_ctx(w, my_rank), H.make_ctx(w, my_rank)]
    ctx_p = H.make_ctx(w, my_rank, max_recv_rows=1)
    recs, toks = _pooled_regions(wr, 5, my_rank, rctx[0], sample_peers=())
    m_rows = sum(rec["n_rows"] for rec in recs)
    cap = max(1, m_rows * min(K, w.experts_per_rank))
    want = ref.dispatch_plain(toks, e2r, my_rank, cap)
    table = B.peers_table(recs, H.DEV)
    n_sets, n_steps = 3, 4
    batches = []
    for b in range(n_sets):
        tk = W.topk_ids(w, 20 + b, my_rank)
        if b == 1:
            tk = tk[: T - 1000].copy()                    # a shorter batch, with a token that goes nowhere
            tk[11, :] = -1
        batches.append((tk, W.payload_rows_pooled(w, 20 + b, my_rank, np.arange(len(tk)))))
    sets = []
    for tk, x in batches:
        sd = B.SendBuffers(rctx[0], T)
        sd.packed.fill_(0x3C)
        sets.append(dict(tk=H.dev(tk), x=H.dev(x), send=sd, recv=B.RecvBuffers(rctx[0], cap)))
    s_send, s_recv = torch.cuda.Stream(), torch.cuda.Stream()
    ev_plan = [torch.cuda.Event(), torch.cuda.Event()]
    no_plan_stats = torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    torch.cuda.synchronize()
    # what the step before the first one leaves behind: index and plan of batch 0
    with torch.cuda.stream(s_recv):
        rctx[0].mw_unpack_index(table, R, cap, sets[0]["recv"].expert_offsets, sets[0]["recv"].stats)
        sd = sets[0]["send"]
        rctx[0].mw_plan(sets[0]["tk"], sd.mask, sd.perm, sd.desc, sd.stats)
        ev_plan[0].record(s_recv)
    ev_steps = []
    for n in range(n_steps):
        s, sn = sets[n % n_sets], sets[(n + 1) % n_sets]
        sd, rv, rn, sdn = s["send"], s["recv"], sn["recv"], sn["send"]
        if schedule == "launch_and_plan":
            with torch.cuda.stream(s_send):
                if n >= 2:
                    s_send.wait_event(ev_steps[n - 2])    # the plan's buffers are those step n - 2 packed from
                ctx_p.mw_plan(sn["tk"], sdn.mask, sdn.perm, sdn.desc, sdn.stats)
                ev_plan[(n + 1) % 2].record(s_send)
            with torch.cuda.stream(s_recv):
                s_recv.wait_event(ev_plan[n % 2])
                rctx[n % 2].mw_stream_step(s["x"], None, s["tk"], sd.perm, sd.stats, sd.packed, sd.row_src_token,
                                           sd.row_topk, R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                                           rv.out_src_token, rctx[(n + 1) % 2], table, R, cap, rn.expert_offsets,
                                           rn.stats, sn["tk"][:0], None, None, None, no_plan_stats)
                ev_steps.append(torch.cuda.Event())
                ev_steps[n].record(s_recv)
        else:
            with torch.cuda.stream(s_recv):
                rctx[n % 2].mw_stream_step(s["x"], None, s["tk"], sd.perm, sd.stats, sd.packed, sd.row_src_token,
                                           sd.row_topk, R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                                           rv.out_src_token, rctx[(n + 1) % 2], table, R, cap, rn.expert_offsets,
                                           rn.stats, sn["tk"], sdn.mask, sdn.perm, sdn.desc, sdn.stats)
    with torch.cuda.stream(s_recv):                       # the batch the last step indexed is expanded, too
        n = n_steps
        rv = sets[n % n_sets]["recv"]
        rctx[n % 2].mw_unpack_expand(R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token)
    torch.cuda.synchronize()
    assert int(no_plan_stats.cpu().numpy().view(B.SEND_STATS_DTYPE)[0]["error_flags"]) == 0
    for b, (s, (tk, x)) in enumerate(zip(sets, batches)):
        g = H.GpuSend.__new__(H.GpuSend)                      # what the steps wrote, in GpuSend's clothes
        g.ctx, g.T, g.buf, g.prefill = rctx[0], len(tk), s["send"], 0x3C
        g.stats = rctx[0].mw_get_send_stats(s["send"].stats)
        g.N, g.G = int(g.stats["n_rows"]), int(g.stats["n_groups"])
        H.check_send(w, g, tk, x, None)
        gs = H.GpuUnpack.__new__(H.GpuUnpack)
        gs.ctx, gs.buf = rctx[0], s["recv"]
        gs.stats = rctx[0].mw_get_recv_stats(s["recv"].stats)
        gs.Q = int(gs.stats["n_out_rows"])
        H.check_unpack(gs, want, "%s: received batch of set %d" % (schedule, b))
    for c in rctx + [ctx_p]:
        c.close()


def test_unpack_in_two_calls_with_two_contexts_in_flight():
    """mw_unpack_index + mw_unpack_expand == mw_unpack; two batches indexed before either is
    expanded (one context each), on two streams with an event between the halves."""
    w = W.scaled(W.C1, n_tokens=150, hidden=512)
    e2r = W.expert_to_rank(w)
    batches = []
    for seed, my_rank in ((1, 3), (2, 40)):
        ctx = H.make_ctx(w, my_rank)
        recs, toks = [], []
        for p in range(w.n_ranks):
            tk = W.topk_ids(w, seed, p)
            x, sc = W.payload_rows(w, seed, p)
            g = H.GpuSend(ctx, tk, x, sc)
            recs.append(H.shrink(g.deliver(my_rank)))
            toks.append((tk, x, sc))
        cap = sum(r["n_rows"] for r in recs) * 4
        batches.append(dict(ctx=ctx, recs=recs, toks=toks, cap=cap, table=B.peers_table(recs, H.DEV),
                            buf=B.RecvBuffers(ctx, cap), my_rank=my_rank))
    s_idx, s_exp = torch.cuda.Stream(), torch.cuda.Stream()
    done = [torch.cuda.Event() for _ in batches]
    torch.cuda.synchronize()
    with torch.cuda.stream(s_idx):
        for b, ev in zip(batches, done):
            b["ctx"].mw_unpack_index(b["table"], w.n_ranks, b["cap"], b["buf"].expert_offsets, b["buf"].stats)
            ev.record(s_idx)
    with torch.cuda.stream(s_exp):
        for b, ev in zip(batches, done):
            s_exp.wait_event(ev)
            b["ctx"].mw_unpack_expand(w.n_ranks, b["buf"].out_rows, None, b["cap"], b["buf"].out_src_peer,
                                      b["buf"].out_src_token)
    torch.cuda.synchronize()
    for b in batches:
        want = ref.dispatch_plain(b["toks"], e2r, b["my_rank"], b["cap"])
        st = b["ctx"].mw_get_recv_stats(b["buf"].stats)
        q = int(st["n_out_rows"])
        assert int(st["error_flags"]) == 0
        H.assert_same_bytes(H.host(b["buf"].expert_offsets), want[4], "two-call expert_offsets")
        H.assert_same_bytes(H.host(b["buf"].out_rows)[:q], want[0], "two-call out_rows")
        H.assert_same_bytes(H.host(b["buf"].out_src_peer)[:q], want[2], "two-call out_src_peer")
        H.assert_same_bytes(H.host(b["buf"].out_src_token)[:q], want[3], "two-call out_src_token")
        one = H.GpuUnpack(b["ctx"], b["recs"], b["cap"])          # the single call, same context
        H.check_unpack(one, want, "single call")
        b["ctx"].close()


def test_index_of_the_next_batch_rides_with_the_expander():
    """A stream of batches through mw_unpack_expand_index_next on two contexts: every batch's
    output must be what mw_unpack gives (bit-exact against the plain definition), whatever ran
    beside its index."""
    for w, my_rank in ((W.scaled(W.C1, n_tokens=150, hidden=512), 3),
                       (W.scaled(W.C2, n_tokens=90, hidden=1024), 40),
                       (W.scaled(W.C3, n_tokens=64, hidden=256), 200)):
        _say("pipelined unpack", w.name)
        e2r = W.expert_to_rank(w)
        ctxs = [H.make_ctx(w, my_rank), H.make_ctx(w, my_rank)]
        batches = []
        for seed in (1, 2, 3, 4):
            recs, toks = [], []
            for p in range(w.n_ranks):
                tk = W.topk_ids(w, seed, p)
                if seed == 3:
                    tk = tk.copy(); tk[::2] = -1                  # a much smaller batch in the middle
                x, sc = W.payload_rows(w, seed, p)
                g = H.GpuSend(ctxs[0], tk, x, sc)
                recs.append(H.shrink(g.deliver(my_rank)))
                toks.append((tk, x, sc))
            cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
            batches.append(dict(recs=recs, toks=toks, cap=cap, table=B.peers_table(recs, H.DEV)))
        bufs = [B.RecvBuffers(ctxs[i % 2], b["cap"]) for i, b in enumerate(batches)]
        R = w.n_ranks
        b0 = batches[0]
        ctxs[0].mw_unpack_index(b0["table"], R, b0["cap"], bufs[0].expert_offsets, bufs[0].stats)
        for i, b in enumerate(batches):
            cur, buf = ctxs[i % 2], bufs[i]
            if i + 1 < len(batches):
                nb, nbuf = batches[i + 1], bufs[i + 1]
                cur.mw_unpack_expand_index_next(R, buf.out_rows, buf.out_scales, b["cap"], buf.out_src_peer,
                                                buf.out_src_token, ctxs[(i + 1) % 2], nb["table"], R, nb["cap"],
                                                nbuf.expert_offsets, nbuf.stats)
            else:
                cur.mw_unpack_expand(R, buf.out_rows, buf.out_scales, b["cap"], buf.out_src_peer, buf.out_src_token)
        torch.cuda.synchronize()
        for i, b in enumerate(batches):
            want = ref.dispatch_plain(b["toks"], e2r, my_rank, b["cap"])
            st = ctxs[i % 2].mw_get_recv_stats(bufs[i].stats)
            q = int(st["n_out_rows"])
            assert int(st["error_flags"]) == 0 and q == len(want[2])
            H.assert_same_bytes(H.host(bufs[i].expert_offsets), want[4], "batch %d expert_offsets" % i)
            H.assert_same_bytes(H.host(bufs[i].out_src_peer)[:q], want[2], "batch %d out_src_peer" % i)
            H.assert_same_bytes(H.host(bufs[i].out_src_token)[:q], want[3], "batch %d out_src_token" % i)
            H.assert_same_bytes(H.host(bufs[i].out_rows)[:q], want[0], "batch %d out_rows" % i)
            if want[1] is not None:
                H.assert_same_bytes(H.host(bufs[i].out_scales)[:q], want[1], "batch %d out_scales" % i)
        with pytest.raises(B.MwError) as ei:                      # one context cannot hold both indexes
            ctxs[0].mw_unpack_expand_index_next(R, bufs[0].out_rows, bufs[0].out_scales, batches[0]["cap"],
                                                bufs[0].out_src_peer, bufs[0].out_src_token, ctxs[0],
                                                batches[1]["table"], R, batches[1]["cap"], bufs[1].expert_offsets,
                                                bufs[1].stats)
        assert ei.value.status == B.MW_ERR_INVALID_ARG
        for c in ctxs:
            c.close()


def _check_plan_outputs(w, ctx, sb, tk, what):
    """mask, perm, descriptors and statistics in `sb` against the oracle's plan of `tk`."""
    e2r = W.expert_to_rank(w)
    m, perm, desc, ost = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
    st = ctx.mw_get_send_stats(sb.stats)
    N, G = int(st["n_rows"]), int(st["n_groups"])
    assert (N, G, int(st["error_flags"])) == (len(perm), len(desc), 0), what
    H.assert_same_bytes(H.host(sb.mask).view(np.uint64)[: len(tk)], m, what + " mask")
    H.assert_same_bytes(H.host(sb.perm)[:N], perm, what + " perm")
    H.assert_same_bytes(H.host(sb.desc).reshape(-1).view(B.DESC_DTYPE)[:G].view(np.uint8), desc.view(np.uint8),
                        what + " desc")
    H.assert_same_bytes(st["rows_per_dest"], ost["rows_per_dest"], what + " rows_per_dest")
    for f in ("multicast_bytes", "unicast_bytes"):
        assert int(st[f]) == int(ost[f]), what + " " + f


@pytest.mark.parametrize("which", ["c1", "c2", "c3", "k12", "one_rank", "wg512", "wg1024"])
def test_plan_of_the_next_batch_rides_with_the_expander(which):
    """A stream of batches through mw_unpack_expand_index_plan_next on two contexts: the receive side
    of every batch against the plain definition, and the riding plan of every next batch -- bitmaps,
    perm, descriptors, statistics -- against the oracle's plan; batch sizes change from call to
    call (one is empty, one has tokens that go nowhere, many tokens share their bitmap), and
    mw_plan itself is used on the same contexts in between."""
    w, my_rank = {"c1": (W.scaled(W.C1, n_tokens=333, hidden=512), 3),
                  "c2": (W.scaled(W.C2, n_tokens=300, hidden=1024), 40),
                  "c3": (W.scaled(W.C3, n_tokens=257, hidden=256), 200),
                  "k12": (W.DispatchWorkload("k12", 22, 130, 260, 12, 200, 256, "bf16", "uniform"), 77),
                  "one_rank": (W.DispatchWorkload("r1", 23, 1, 4, 2, 130, 256, "bf16", "uniform"), 0),
                  # rows of 462 and 1001 chunks: the launch's workgroups have 512 and 1024 lanes
                  "wg512": (W.DispatchWorkload("wg512", 24, 8, 16, 2, 140, 7168, "fp8", "uniform"), 5),
                  "wg1024": (W.DispatchWorkload("wg1024", 25, 8, 16, 3, 140, 8008, "bf16", "uniform"), 2)}[which]
    _say("riding plan", w.name)
    e2r = W.expert_to_rank(w)
    ctxs = [H.make_ctx(w, my_rank, max_tokens=1200), H.make_ctx(w, my_rank, max_tokens=1200)]
    R = w.n_ranks
    batches = []
    for seed in (1, 2, 3, 4, 5):
        recs, toks = [], []
        for p in range(R):
            tk = W.topk_ids(w, seed, p)
            x, sc = W.payload_rows(w, seed, p)
            recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, sc).deliver(my_rank)))
            toks.append((tk, x, sc))
        cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
        batches.append(dict(recs=recs, toks=toks, cap=cap, table=B.peers_table(recs, H.DEV)))
    # the send-side batches whose plans ride along: sizes and contents vary
    wide = W.scaled(w, n_tokens=1200)
    sends = [W.topk_ids(w, 11, my_rank), W.topk_ids(wide, 12, my_rank), np.zeros((0, w.top_k), np.int32),
             W.topk_ids(wide, 14, my_rank)[:700].copy(), W.topk_ids(w, 15, my_rank)[:65].copy()]
    sends[1][::5] = -1                                     # tokens that go nowhere
    sends[3][100:600] = sends[3][99]                       # one long run of equal bitmaps
    sbufs = [B.SendBuffers(ctxs[0], 1200) for _ in sends]
    bufs = [B.RecvBuffers(ctxs[i % 2], b["cap"]) for i, b in enumerate(batches)]
    b0 = batches[0]
    ctxs[0].mw_unpack_index(b0["table"], R, b0["cap"], bufs[0].expert_offsets, bufs[0].stats)
    for i, b in enumerate(batches):
        cur, buf = ctxs[i % 2], bufs[i]
        nb, nbuf = batches[(i + 1) % len(batches)], bufs[(i + 1) % len(batches)]
        tk_d = H.dev(sends[i]) if len(sends[i]) else torch.zeros((0, w.top_k), dtype=torch.int32, device=H.DEV)
        if i + 1 < len(batches):
            cur.mw_unpack_expand_index_plan_next(R, buf.out_rows, buf.out_scales, b["cap"], buf.out_src_peer,
                                                 buf.out_src_token, ctxs[(i + 1) % 2], nb["table"], R, nb["cap"],
                                                 nbuf.expert_offsets, nbuf.stats, tk_d, sbufs[i].mask, sbufs[i].perm,
                                                 sbufs[i].desc, sbufs[i].stats)
        else:
            cur.mw_unpack_expand(R, buf.out_rows, buf.out_scales, b["cap"], buf.out_src_peer, buf.out_src_token)
            cur.mw_plan(tk_d, sbufs[i].mask, sbufs[i].perm, sbufs[i].desc, sbufs[i].stats)
        if i == 1:                                         # the two-kernel plan on the context the next ride uses
            ctxs[(i + 2) % 2].mw_plan(H.dev(sends[0]), sbufs[0].mask, sbufs[0].perm, sbufs[0].desc, sbufs[0].stats)
    torch.cuda.synchronize()
    for i, b in enumerate(batches):
        want = ref.dispatch_plain(b["toks"], e2r, my_rank, b["cap"])
        st = ctxs[i % 2].mw_get_recv_stats(bufs[i].stats)
        q = int(st["n_out_rows"])
        assert int(st["error_flags"]) == 0 and q == len(want[2])
        H.assert_same_bytes(H.host(bufs[i].expert_offsets), want[4], "batch %d expert_offsets" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_peer)[:q], want[2], "batch %d out_src_peer" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_token)[:q], want[3], "batch %d out_src_token" % i)
        H.assert_same_bytes(H.host(bufs[i].out_rows)[:q], want[0], "batch %d out_rows" % i)
        if want[1] is not None:
            H.assert_same_bytes(H.host(bufs[i].out_scales)[:q], want[1], "batch %d out_scales" % i)
    for i, tk in enumerate(sends):
        _check_plan_outputs(w, ctxs[0], sbufs[i], tk, "riding plan %d" % i)
    with pytest.raises(B.MwError) as ei:                          # more tokens than the context was made for
        big = torch.zeros((1201, w.top_k), dtype=torch.int32, device=H.DEV)
        ctxs[0].mw_unpack_expand_index_plan_next(R, bufs[0].out_rows, bufs[0].out_scales, batches[0]["cap"],
                                                 bufs[0].out_src_peer, bufs[0].out_src_token, ctxs[1],
                                                 batches[1]["table"], R, batches[1]["cap"], bufs[1].expert_offsets,
                                                 bufs[1].stats, big, sbufs[0].mask, sbufs[0].perm, sbufs[0].desc,
                                                 sbufs[0].stats)
    assert ei.value.status == B.MW_ERR_CAPACITY
    for c in ctxs:
        c.close()


@pytest.mark.parametrize("which", ["c1", "c3"])
def test_riding_plan_at_full_batch_size(which):
    """The plan of a full-size batch (C1: 4096 tokens over 64 ranks; C3: 8192 tokens over 256
    ranks, short keys) riding with the expander of a small batch: several slices per token, many
    finishing workgroups; twice in a row on alternating contexts."""
    base = W.C1 if which == "c1" else W.C3
    w = W.scaled(base, hidden=1024 if which == "c1" else 256)
    small = W.scaled(w, n_tokens=64)
    my_rank = 3
    _say("riding plan, full batch", w.name, "T", w.n_tokens)
    ctxs = [H.make_ctx(w, my_rank, max_recv_rows=4096), H.make_ctx(w, my_rank, max_recv_rows=4096)]
    recs = []
    for p in range(2):
        tk = W.topk_ids(small, 1, p)
        x, sc = W.payload_rows(small, 1, p)
        tk[::2, 0] = my_rank * small.experts_per_rank             # make sure something arrives
        recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, sc).deliver(my_rank)))
    cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
    table = B.peers_table(recs, H.DEV)
    bufs = [B.RecvBuffers(ctxs[0], cap), B.RecvBuffers(ctxs[1], cap)]
    ctxs[0].mw_unpack_index(table, 2, cap, bufs[0].expert_offsets, bufs[0].stats)
    sends = [W.topk_ids(w, 21, my_rank), W.topk_ids(w, 22, my_rank)]
    sends[1][::9] = -1
    sbufs = [B.SendBuffers(ctxs[0], w.n_tokens) for _ in sends]
    for i, tk in enumerate(sends):
        cur, nxt = ctxs[i % 2], ctxs[(i + 1) % 2]
        cur.mw_unpack_expand_index_plan_next(2, bufs[i % 2].out_rows, bufs[i % 2].out_scales, cap,
                                             bufs[i % 2].out_src_peer, bufs[i % 2].out_src_token, nxt, table, 2, cap,
                                             bufs[(i + 1) % 2].expert_offsets, bufs[(i + 1) % 2].stats, H.dev(tk),
                                             sbufs[i].mask, sbufs[i].perm, sbufs[i].desc, sbufs[i].stats)
    torch.cuda.synchronize()
    for i, tk in enumerate(sends):
        _check_plan_outputs(w, ctxs[0], sbufs[i], tk, "full-size riding plan %d" % i)
    for c in ctxs:
        c.close()


@pytest.mark.parametrize("which", ["c1", "c2", "c3", "wg1024"])
def test_stream_step_packs_expands_indexes_and_plans_in_one_launch(which):
    """mw_stream_step over a stream of batches on two contexts: in step i the batch planned by
    step i - 1 is packed, received batch i is expanded, received batch i + 1 indexed, and the
    batch after that planned.  Every output of every step against the oracle / the plain definition."""
    w, my_rank = {"c1": (W.scaled(W.C1, n_tokens=333, hidden=512), 3),
                  "c2": (W.scaled(W.C2, n_tokens=300, hidden=1024), 40),
                  "c3": (W.scaled(W.C3, n_tokens=257, hidden=256), 200),
                  "wg1024": (W.DispatchWorkload("wg1024", 25, 8, 16, 3, 140, 8008, "bf16", "uniform"), 2)}[which]
    _say("stream step", w.name)
    e2r = W.expert_to_rank(w)
    T, R = w.n_tokens, w.n_ranks
    ctxs = [H.make_ctx(w, my_rank), H.make_ctx(w, my_rank)]
    n_steps = 4
    batches = []                                           # what this rank receives in step i
    for seed in range(1, n_steps + 2):
        recs, toks = [], []
        for p in range(R):
            tk = W.topk_ids(w, seed, p)
            x, sc = W.payload_rows(w, seed, p)
            recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, sc).deliver(my_rank)))
            toks.append((tk, x, sc))
        cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
        batches.append(dict(recs=recs, toks=toks, cap=cap, table=B.peers_table(recs, H.DEV)))
    sends = []                                             # what this rank sends: batch j is planned in step j - 1
    for j in range(n_steps + 1):
        tk = W.topk_ids(w, 30 + j, my_rank)
        if j == 2:
            tk[::3] = -1                                   # fewer rows than tokens
        x, sc = W.payload_rows(w, 30 + j, my_rank)
        sends.append(dict(tk=tk, x=x, sc=sc, tk_d=H.dev(tk), x_d=H.dev(x), s_d=H.dev(sc), buf=B.SendBuffers(ctxs[0], T)))
    bufs = [B.RecvBuffers(ctxs[i % 2], b["cap"]) for i, b in enumerate(batches)]
    # before the first step: the plan of send batch 0 and the index of received batch 0
    s0 = sends[0]
    ctxs[0].mw_plan(s0["tk_d"], s0["buf"].mask, s0["buf"].perm, s0["buf"].desc, s0["buf"].stats)
    ctxs[0].mw_unpack_index(batches[0]["table"], R, batches[0]["cap"], bufs[0].expert_offsets, bufs[0].stats)
    for i in range(n_steps):
        cur, nxt = ctxs[i % 2], ctxs[(i + 1) % 2]
        sd, sn = sends[i], sends[i + 1]
        b, nb = batches[i], batches[i + 1]
        cur.mw_stream_step(sd["x_d"], sd["s_d"], sd["tk_d"], sd["buf"].perm, sd["buf"].stats, sd["buf"].packed,
                           sd["buf"].row_src_token, sd["buf"].row_topk, R, bufs[i].out_rows, bufs[i].out_scales,
                           b["cap"], bufs[i].out_src_peer, bufs[i].out_src_token, nxt, nb["table"], R, nb["cap"],
                           bufs[i + 1].expert_offsets, bufs[i + 1].stats, sn["tk_d"], sn["buf"].mask, sn["buf"].perm,
                           sn["buf"].desc, sn["buf"].stats)
    torch.cuda.synchronize()
    for i in range(n_steps):
        b = batches[i]
        want = ref.dispatch_plain(b["toks"], e2r, my_rank, b["cap"])
        st = ctxs[i % 2].mw_get_recv_stats(bufs[i].stats)
        q = int(st["n_out_rows"])
        assert int(st["error_flags"]) == 0 and q == len(want[2])
        H.assert_same_bytes(H.host(bufs[i].expert_offsets), want[4], "step %d expert_offsets" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_peer)[:q], want[2], "step %d out_src_peer" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_token)[:q], want[3], "step %d out_src_token" % i)
        H.assert_same_bytes(H.host(bufs[i].out_rows)[:q], want[0], "step %d out_rows" % i)
        if want[1] is not None:
            H.assert_same_bytes(H.host(bufs[i].out_scales)[:q], want[1], "step %d out_scales" % i)
    for j in range(n_steps + 1):
        sd = sends[j]
        _check_plan_outputs(w, ctxs[0], sd["buf"], sd["tk"], "send batch %d" % j)
        if j < n_steps:                                    # packed in step j
            _, perm, _, _ = ref.plan(sd["tk"], e2r, R, w.row_bytes)
            packed, src, rtk = ref.pack(sd["x"], sd["sc"], sd["tk"], perm)
            n = len(perm)
            H.assert_same_bytes(H.host(sd["buf"].packed)[:n], packed, "send batch %d packed rows" % j)
            H.assert_same_bytes(H.host(sd["buf"].row_src_token)[:n], src, "send batch %d row_src_token" % j)
            H.assert_same_bytes(H.host(sd["buf"].row_topk)[:n], rtk, "send batch %d row_topk" % j)
    for c in ctxs:
        c.close()


def test_unpack_after_a_smaller_batch_strides_over_the_rows():
    """The expander's launch is sized from the row count seen at the last mw_get_recv_stats; a later,
    larger batch on the same context must still be expanded completely (and a smaller one too)."""
    w = W.scaled(W.C1, n_tokens=300, hidden=256)
    e2r = W.expert_to_rank(w)
    my_rank = 9
    ctx = H.make_ctx(w, my_rank)
    recs, toks = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, 7, p)
        x, sc = W.payload_rows(w, 7, p)
        g = H.GpuSend(ctx, tk, x, sc)
        recs.append(H.shrink(g.deliver(my_rank)))
        toks.append((tk, x, sc))
    empty = [(np.full_like(t[0], -1), t[1], t[2]) for t in toks]
    few = [dict(r, n_desc=0, n_rows=0) for r in recs]
    few[5] = recs[5]
    cap = sum(r["n_rows"] for r in recs) * 4
    small = H.GpuUnpack(ctx, few, cap)                     # reads the statistics: the hint is now tiny
    H.check_unpack(small, ref.dispatch_plain(empty[:5] + [toks[5]] + empty[6:], e2r, my_rank, cap), "one peer")
    assert int(small.stats["n_rows_seen"]) == recs[5]["n_rows"]
    big = H.GpuUnpack(ctx, recs, cap)                      # ~60 times as many rows as the hint
    H.check_unpack(big, ref.dispatch_plain(toks, e2r, my_rank, cap), "all peers after one peer")
    assert int(big.stats["n_rows_seen"]) == sum(r["n_rows"] for r in recs)
    again = H.GpuUnpack(ctx, few, cap)                     # and back
    H.check_unpack(again, ref.dispatch_plain(empty[:5] + [toks[5]] + empty[6:], e2r, my_rank, cap), "one peer again")
    ctx.close()


# ------------------------------------------------------------------ AllGather
@pytest.mark.parametrize("w", [W.AllGatherWorkload("ag_small", 41, 8, 1000 * 8), W.C4],
                         ids=["small", "C4_full"])
def test_allgather(w):
    _say("allgather", w.name)
    ctx = B.Context(w.n_ranks, 0, 1, w.my_rank, 0, B.MW_ROW_BYTES, 1, 0, None, row_bytes=w.shard_bytes,
                    device=H.DEV)
    shards = [W.allgather_shard(w, W.BASE_SEED, r) for r in range(w.n_ranks)]
    desc = torch.zeros(B.DESC_BYTES, dtype=torch.uint8, device=H.DEV)
    stats = torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    ctx.mw_plan_allgather(w.shard_bytes, desc, stats)
    od, ost = ref.plan_allgather(w.n_ranks, w.shard_bytes)
    H.assert_same_bytes(H.host(desc), od.view(np.uint8).reshape(-1), "allgather desc")
    st = ctx.mw_get_send_stats(stats)
    H.assert_same_bytes(np.array([st]).view(np.uint8), np.array([ost]).view(np.uint8), "allgather stats")
    mine = H.dev(shards[w.my_rank])
    send = torch.zeros_like(mine)
    ctx.mw_pack_allgather(mine, w.shard_bytes, send)
    H.assert_same_bytes(H.host(send), ref.pack_allgather(shards[w.my_rank]).view(np.uint16), "send buffer")
    recv = [send if r == w.my_rank else H.dev(shards[r]) for r in range(w.n_ranks)]
    table = torch.tensor([t.data_ptr() for t in recv], dtype=torch.int64, device=H.DEV)
    out = torch.zeros(w.n_ranks * w.shard_elems, dtype=torch.int16, device=H.DEV)
    ctx.mw_unpack_allgather(table, w.shard_bytes, out)
    torch.cuda.synchronize()
    H.assert_same_bytes(H.host(out).view(np.uint8), ref.unpack_allgather(shards), "gathered output")
    # the same three as one launch (mw_allgather_step): the received shards of one operation are
    # assembled while the shard of the next one (here: another rank's data) is loaded and planned
    nxt = W.allgather_shard(w, W.BASE_SEED + 1, w.my_rank)
    nxt_d, send2 = H.dev(nxt), torch.zeros_like(mine)
    desc.zero_(); stats.zero_(); out.zero_()
    ctx.mw_allgather_step(nxt_d, w.shard_bytes, send2, desc, stats, table, out)
    torch.cuda.synchronize()
    H.assert_same_bytes(H.host(out).view(np.uint8), ref.unpack_allgather(shards), "step: gathered output")
    H.assert_same_bytes(H.host(send2), ref.pack_allgather(nxt).view(np.uint16), "step: send buffer")
    H.assert_same_bytes(H.host(desc), od.view(np.uint8).reshape(-1), "step: desc")
    H.assert_same_bytes(np.array([ctx.mw_get_send_stats(stats)]).view(np.uint8), np.array([ost]).view(np.uint8),
                        "step: stats")
    # an empty shard: nothing moves, the plan is the oracle's plan of zero bytes
    desc.zero_(); stats.zero_()
    before = H.host(out).copy()
    ctx.mw_allgather_step(None, 0, None, desc, stats, None, None)
    torch.cuda.synchronize()
    od0, ost0 = ref.plan_allgather(w.n_ranks, 0)
    H.assert_same_bytes(H.host(desc), od0.view(np.uint8).reshape(-1), "step, empty shard: desc")
    H.assert_same_bytes(np.array([ctx.mw_get_send_stats(stats)]).view(np.uint8), np.array([ost0]).view(np.uint8),
                        "step, empty shard: stats")
    H.assert_same_bytes(H.host(out), before, "step, empty shard: output untouched")
    # argument errors are returned, nothing is launched
    for args, want in [((nxt_d, w.shard_bytes - 8, send2, desc, stats, table, out), B.MW_ERR_UNSUPPORTED),
                       ((nxt_d, -16, send2, desc, stats, table, out), B.MW_ERR_INVALID_ARG),
                       ((None, w.shard_bytes, send2, desc, stats, table, out), B.MW_ERR_INVALID_ARG),
                       ((nxt_d, w.shard_bytes, send2, desc, stats, None, out), B.MW_ERR_INVALID_ARG),
                       ((nxt_d, w.shard_bytes, send2, None, stats, table, out), B.MW_ERR_INVALID_ARG)]:
        with pytest.raises(B.MwError) as ei:
            ctx.mw_allgather_step(*args)
        assert ei.value.status == want
    ctx.close()


@pytest.mark.parametrize("direct_frac", [0.0, 0.5, 0.75, 1.0])
@pytest.mark.parametrize("w", [W.AllGatherWorkload("ag_small", 41, 8, 1000 * 8), W.C4], ids=["small", "C4_full"])
def test_allgather_split_fragment(w, direct_frac):
    """Section 5.2: fragment split into a direct and a relayed segment; the assembly of the two
    pieces of every rank equals the plain AllGather result."""
    _say("allgather split", w.name, direct_frac)
    s = w.shard_bytes
    if 0.0 < direct_frac < 1.0:      # bandwidth ratio that puts this fraction on the direct path
        direct = B.mw_allgather_split_point(s, direct_frac, 1.0 - direct_frac, 1)
        assert direct == ref.allgather_split_point(s, direct_frac, 1.0 - direct_frac, 1)
    else:
        direct = int(direct_frac) * s
    ctx = B.Context(w.n_ranks, 0, 1, w.my_rank, 0, B.MW_ROW_BYTES, 1, 0, None, row_bytes=s, device=H.DEV)
    desc = torch.zeros(2 * B.DESC_BYTES, dtype=torch.uint8, device=H.DEV)
    stats = torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    ctx.mw_plan_allgather_split(s, direct, desc, stats)
    od, ost = ref.plan_allgather_split(w.n_ranks, s, direct)
    H.assert_same_bytes(H.host(desc), od.view(np.uint8).reshape(-1), "split desc pair")
    st = ctx.mw_get_send_stats(stats)
    H.assert_same_bytes(np.array([st]).view(np.uint8), np.array([ost]).view(np.uint8), "split stats")
    shards = [W.allgather_shard(w, W.BASE_SEED, r).view(np.uint8) for r in range(w.n_ranks)]
    dp = [H.dev(np.ascontiguousarray(x[:direct])) if direct else None for x in shards]
    rp = [H.dev(np.ascontiguousarray(x[direct:])) if direct < s else None for x in shards]
    dt = torch.tensor([0 if t is None else t.data_ptr() for t in dp], dtype=torch.int64, device=H.DEV)
    rt = torch.tensor([0 if t is None else t.data_ptr() for t in rp], dtype=torch.int64, device=H.DEV)
    out = torch.zeros(w.n_ranks * s, dtype=torch.uint8, device=H.DEV)
    ctx.mw_unpack_allgather_split(dt, rt, s, direct, out)
    torch.cuda.synchronize()
    want = ref.unpack_allgather_split([x[:direct] for x in shards], [x[direct:] for x in shards], s, direct)
    H.assert_same_bytes(H.host(out), want, "split assembly")
    H.assert_same_bytes(H.host(out), ref.unpack_allgather(shards), "split assembly vs plain AllGather")
    ctx.close()


def test_allgather_equals_dispatch_with_all_ranks_set():
    # Section 2.3.3 / 5.2: AllGather is the static destination set "everyone"
    R, elems = 8, 2048
    w = W.AllGatherWorkload("ag_as_dispatch", 42, R, elems)
    shards = [W.allgather_shard(w, 5, r) for r in range(R)]
    e2r = np.arange(R, dtype=np.int32)
    ctx = B.Context(R, R, R, 3, elems, B.MW_ROW_BF16, 1, R, e2r, device=H.DEV)
    tk = np.arange(R, dtype=np.int32).reshape(1, R)
    recs = []
    for p in range(R):
        g = H.GpuSend(ctx, tk, shards[p].reshape(1, -1), None)
        recs.append(H.shrink(g.deliver(3)))
    gu = H.GpuUnpack(ctx, recs, R)
    H.assert_same_bytes(gu.host_out()[0].reshape(-1), np.concatenate(shards).view(np.uint8), "dispatch as allgather")
    ctx.close()


# ------------------------------------------------------------------ edge and degenerate cases
def _small(fmt="bf16", T=64, K=2, R=8, E=16, H_=256):
    return W.DispatchWorkload("edge", 77, R, E, K, T, H_, fmt, "uniform")


def test_empty_batch_and_tokens_without_experts():
    w = _small()
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, 0)
    g = H.GpuSend(ctx, np.zeros((0, 2), np.int32), np.zeros((0, w.hidden), np.uint16), None)
    assert (g.N, g.G, int(g.stats["unicast_bytes"]), int(g.stats["error_flags"])) == (0, 0, 0, 0)
    tk = np.full((w.n_tokens, 2), -1, dtype=np.int32)
    x, _ = W.payload_rows(w, 1, 0)
    g = H.GpuSend(ctx, tk, x, None)
    assert (g.N, g.G) == (0, 0)
    tk[10] = (3, -1); tk[40] = (-1, 2)
    g = H.GpuSend(ctx, tk, x, None)
    H.check_send(w, g, tk, x, None)
    assert g.N == 2
    # unpack of peers that sent nothing
    rec = H.shrink(H.GpuSend(ctx, np.full((4, 2), -1, np.int32), x[:4], None).deliver(0))
    gu = H.GpuUnpack(ctx, [rec, rec], 4)
    assert gu.Q == 0 and int(gu.stats["error_flags"]) == 0
    assert H.host(gu.buf.expert_offsets).tolist() == [0, 0, 0]
    ctx.close()


def test_all_masks_equal_single_group_is_memcpy():
    w = _small(T=300)
    tk = np.tile(np.array([[5, 0]], dtype=np.int32), (w.n_tokens, 1))
    x, _ = W.payload_rows(w, 1, 0)
    ctx = H.make_ctx(w, 0)
    g = H.GpuSend(ctx, tk, x, None)
    H.check_send(w, g, tk, x, None)
    assert g.G == 1
    H.assert_same_bytes(g.host_pack()[0].reshape(-1), x.view(np.uint8).reshape(-1), "packed == input")
    ctx.close()


def test_single_destination_is_plain_alltoallv():
    # Section 4.3.3 rule 2: one destination -> a plain write; the plan is a stable sort by rank
    w = _small(T=500, K=1, R=16, E=32)
    run_dispatch(w, 3, 9)
    tk = W.topk_ids(w, 3, 0)
    x, _ = W.payload_rows(w, 3, 0)
    ctx = H.make_ctx(w, 0)
    g = H.GpuSend(ctx, tk, x, None)
    dest = W.expert_to_rank(w)[tk[:, 0]]
    assert np.array_equal(g.host_plan()[1], np.argsort(dest, kind="stable"))
    assert int(g.stats["unicast_bytes"]) == int(g.stats["multicast_bytes"])
    ctx.close()


def test_duplicate_ids_and_padding_inside_tokens():
    w = _small(T=96, K=4)
    tk = W.topk_ids(w, 8, 2)
    tk[::3, 1] = tk[::3, 0]          # duplicate expert
    tk[1::5, 3] = -1                 # padding
    x, _ = W.payload_rows(w, 8, 2)
    for my_rank in (0, 7):
        e2r = W.expert_to_rank(w)
        ctx = H.make_ctx(w, my_rank)
        g = H.GpuSend(ctx, tk, x, None)
        perm, desc, packed, src, rtk = H.check_send(w, g, tk, x, None)
        rec = H.shrink(g.deliver(my_rank))
        o1 = ref.dispatch_plain([(tk, x, None)], e2r, my_rank, 4 * w.n_tokens)
        gu = H.GpuUnpack(ctx, [rec], 4 * w.n_tokens)
        H.check_unpack(gu, o1)
        ctx.close()


def test_more_than_eight_local_experts_per_row():
    # 2 ranks x 20 experts, 24 ids per token: a row goes to up to 20 experts of one rank, so the
    # hit slots beyond the eight kept in registers are used; 64 ids per token is the maximum
    run_dispatch(W.DispatchWorkload("dense20", 91, 2, 40, 24, 100, 256, "bf16", "uniform"), 1, 1, also_full=True)
    run_dispatch(W.DispatchWorkload("k64", 92, 4, 128, 64, 60, 128, "bf16", "uniform"), 2, 3)
    run_dispatch(W.DispatchWorkload("k64_fp8", 93, 4, 128, 64, 40, 512, "fp8", "uniform"), 3, 0)


def test_more_rows_than_one_launch_has_workgroup_rows():
    # 20000 tokens per rank, narrow rows: more than 32768 received rows (the row movers' grids
    # stop there and stride) and 79 token blocks in the plan
    w = W.DispatchWorkload("long", 94, 4, 8, 2, 20000, 64, "bf16", "uniform")
    gu = run_dispatch(w, 1, 2, tier2=False)
    assert int(gu.stats["n_recv_rows"]) > 32768
    # 30000 tokens and 20 local experts: the experts' source-token bitmaps no longer fit in LDS
    # together, so the receive index makes several passes over the rows
    w = W.DispatchWorkload("long_many_experts", 96, 2, 40, 4, 30000, 32, "bf16", "uniform")
    run_dispatch(w, 2, 1, tier2=False, check_all_senders=False)


@pytest.mark.parametrize("T,R,E,K", [(8193, 64, 256, 8), (9000, 256, 256, 8), (40000, 64, 128, 4), (65536, 130, 260, 8),
                                     (65536, 8, 8, 2), (9500, 256, 512, 12)])
def test_plan_of_large_batches(T, R, E, K):
    """Batches the plan orders through sorted chunks (and, with 12 ids per token over 256 ranks,
    one that still takes the all-pairs walk): bitmaps, perm, descriptors and statistics against
    the oracle; some tokens go nowhere, many share their bitmap."""
    _say("large plan", T, R, E, K)
    w = W.DispatchWorkload("large", 95, R, E, K, T, 8, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    tk = W.topk_ids(w, 3, 0)
    tk[::97] = -1
    tk[5::11, K - 1] = -1
    if R == 8:
        tk[1000:30000] = tk[999]                      # one long run of equal bitmaps across many chunks
    ctx = H.make_ctx(w, 0, max_recv_rows=1)
    tk_d = H.dev(tk)
    sb = B.SendBuffers(ctx, T)
    for _ in range(2):                                   # twice: the plan leaves its counters clean
        ctx.mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
    st = ctx.mw_get_send_stats(sb.stats)
    m, perm, desc, ost = ref.plan(tk, e2r, R, w.row_bytes)
    N, G = int(st["n_rows"]), int(st["n_groups"])
    assert (N, G, int(st["error_flags"])) == (len(perm), len(desc), 0)
    H.assert_same_bytes(H.host(sb.mask).view(np.uint64), m, "mask")
    H.assert_same_bytes(H.host(sb.perm)[:N], perm, "perm")
    H.assert_same_bytes(H.host(sb.desc).reshape(-1).view(B.DESC_DTYPE)[:G].view(np.uint8), desc.view(np.uint8), "desc")
    H.assert_same_bytes(st["rows_per_dest"], ost["rows_per_dest"], "rows_per_dest")
    assert int(st["unicast_bytes"]) == int(ost["unicast_bytes"])
    # and a small batch afterwards on the same context (the other ordering path, same counters)
    small = tk[:300].copy()
    ctx.mw_plan(H.dev(small), sb.mask, sb.perm, sb.desc, sb.stats)
    st = ctx.mw_get_send_stats(sb.stats)
    m, perm, desc, ost = ref.plan(small, e2r, R, w.row_bytes)
    assert (int(st["n_rows"]), int(st["n_groups"])) == (len(perm), len(desc))
    H.assert_same_bytes(H.host(sb.perm)[: len(perm)], perm, "perm after a large batch")
    ctx.close()


def test_invalid_expert_ids_set_the_error_flag():
    w = _small()
    tk = W.topk_ids(w, 1, 0)
    x, _ = W.payload_rows(w, 1, 0)
    bad = tk.copy(); bad[7, 1] = w.n_experts; bad[20, 0] = -5
    ctx = H.make_ctx(w, 0)
    g = H.GpuSend(ctx, bad, x, None)
    assert int(g.stats["error_flags"]) & B.MW_FLAG_BAD_EXPERT
    with pytest.raises(ref.OracleError):
        ref.plan(bad, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    # the bad entries are ignored: same plan as with -1 in their place
    ign = bad.copy(); ign[7, 1] = -1; ign[20, 0] = -1
    m, perm, desc, st = ref.plan(ign, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    H.assert_same_bytes(g.host_plan()[1], perm, "perm with ignored ids")
    # the flag does not stick to the next call
    g = H.GpuSend(ctx, tk, x, None)
    assert int(g.stats["error_flags"]) == 0
    ctx.close()


def test_output_capacity_overflow_is_flagged_and_bounded():
    w = _small(T=128)
    ctx = H.make_ctx(w, 0)
    recs, toks, bufs = [], [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, 2, p); x, _ = W.payload_rows(w, 2, p)
        recs.append(H.shrink(H.GpuSend(ctx, tk, x, None).deliver(0)))
        toks.append((tk, x, None))
        bufs.append(ref.deliver(*H.oracle_send(w, tk, x, None), 0))
    o1 = ref.dispatch_plain(toks, W.expert_to_rank(w), 0, 10 ** 6)
    Q = len(o1[2])
    cap = Q // 2
    gu = H.GpuUnpack(ctx, recs, cap)
    assert int(gu.stats["error_flags"]) & B.MW_FLAG_OUT_CAPACITY and gu.Q == Q
    got = gu.host_out()
    H.assert_same_bytes(got[0], o1[0][:cap], "rows below capacity are still exact")
    with pytest.raises(ref.OracleError):
        ref.unpack(bufs, w.top_k, W.expert_to_rank(w), 0, w.row_bytes, 0, cap)
    ctx.close()


def test_host_side_argument_errors():
    lib = B.load()
    w = _small()
    with pytest.raises(B.MwError) as ei:
        B.Context(300, 16, 2, 0, 256, B.MW_ROW_BF16, 8, 8, np.zeros(16, np.int32), device=H.DEV)
    assert ei.value.status == B.MW_ERR_UNSUPPORTED
    with pytest.raises(B.MwError) as ei:
        B.Context(8, 16, 2, 0, 256, B.MW_ROW_FP8_E4M3_BLOCK128, 8, 8, W.expert_to_rank(w), device=H.DEV)
    assert ei.value.status == B.MW_ERR_UNSUPPORTED          # fp8 rows need H % 512 == 0
    with pytest.raises(B.MwError) as ei:
        B.Context(8, 16, 2, 9, 256, B.MW_ROW_BF16, 8, 8, W.expert_to_rank(w), device=H.DEV)
    assert ei.value.status == B.MW_ERR_INVALID_ARG
    ctx = H.make_ctx(w, 0, max_tokens=16)
    tk = H.dev(W.topk_ids(w, 1, 0))
    sb = B.SendBuffers(ctx, w.n_tokens)
    with pytest.raises(B.MwError) as ei:
        ctx.mw_plan(tk, sb.mask, sb.perm, sb.desc, sb.stats)
    assert ei.value.status == B.MW_ERR_CAPACITY
    assert lib.mw_plan(None, None, 0, None, None, None, None, None) == B.MW_ERR_INVALID_ARG
    ctx.close()


# ------------------------------------------------------------------ row sizes across the launch shapes
@pytest.mark.parametrize("hidden", [8, 24, 520, 5120, 5128, 5184, 8200, 16392])
def test_row_sizes_across_launch_shapes(hidden):
    """Rows of 1, 3, 65, 640, 641, 648, 1025 and 2049 16-byte chunks: a single partial wave, just
    over one wave, the largest one-workgroup row, the first sizes beyond it (cut into single waves
    only when the row is whole cache lines), and rows longer than one 1024-lane workgroup."""
    w = W.DispatchWorkload("rows", 91, 8, 16, 3, 70, hidden, "bf16", "uniform")
    run_dispatch(w, 4, 2, also_full=True)


def test_opaque_byte_rows():
    """MW_ROW_BYTES with experts: the rows are bytes of any meaning (here 1040 of them)."""
    R, E, K, T, rb, my_rank = 8, 24, 4, 150, 1040, 5
    w = W.DispatchWorkload("bytes", 92, R, E, K, T, rb // 2, "bf16", "uniform")     # routing and sizes only
    e2r = W.expert_to_rank(w)
    ctx = B.Context(R, E, K, my_rank, 0, B.MW_ROW_BYTES, T, R * T, e2r, row_bytes=rb, device=H.DEV)
    assert ctx.row_bytes == rb
    rng = np.random.default_rng(92)
    toks, recs = [], []
    for p in range(R):
        tk = W.topk_ids(w, 6, p)
        x = rng.integers(0, 256, size=(T, rb), dtype=np.uint8)
        toks.append((tk, x, None))
        g = H.GpuSend(ctx, tk, x, None)
        H.check_send(w, g, tk, x, None)
        recs.append(H.shrink(g.deliver(my_rank)))
    cap = sum(r["n_rows"] for r in recs) * min(K, E // R)
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, ref.dispatch_plain(toks, e2r, my_rank, cap), "opaque rows")
    ctx.close()


# ------------------------------------------------------------------ rows further apart than they are long
@pytest.mark.parametrize("which", ["fp8", "bf16_odd", "c0"])
def test_row_stride(which):
    """mw_config.row_stride_bytes: packed, delivered and received rows start a stride apart (fp8 rows
    of 1056 bytes every 1152, the next multiple of 128; bf16 rows of 1040 bytes every 1280; C0's rows
    of 512 bytes every 528).  Every output is what it is with rows back to back, the bytes between
    rows stay untouched, and mw_stream_step packs and expands with the same stride."""
    w, stride, my_rank = {"fp8": (W.scaled(W.C2, n_tokens=200, hidden=1024), 1152, 9),
                          "bf16_odd": (W.DispatchWorkload("odd", 96, 8, 16, 3, 150, 520, "bf16", "uniform"), 1280, 2),
                          "c0": (W.C0, 528, 5)}[which]
    assert stride > w.row_bytes
    run_dispatch(w, 3, my_rank, also_full=True, stream_step=True, row_stride=stride)
