"""GPU parity of the packet path (bitmap and row metadata in front of every row, Section 6.4):
mw_pack_packets and mw_unpack_packets, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Bit-exact."""
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


class GpuPackets:
    """mw_plan + mw_pack_packets of one rank's tokens."""

    def __init__(self, ctx, topk, x, scales, x_dev=None, scales_dev=None):
        self.ctx, self.T = ctx, topk.shape[0]
        self.topk_d = H.dev(topk.astype(np.int32))
        self.x_d = x_dev if x_dev is not None else H.dev(x)
        self.s_d = scales_dev if scales_dev is not None else H.dev(scales)
        self.buf = B.SendBuffers(ctx, self.T)
        self.hb = B.mw_packet_header_bytes(ctx.top_k)
        self.packets = torch.zeros((max(self.T, 1), self.hb + ctx.row_bytes), dtype=torch.uint8, device=H.DEV)
        ctx.mw_plan(self.topk_d, self.buf.mask, self.buf.perm, self.buf.desc, self.buf.stats)
        ctx.mw_pack_packets(self.x_d, self.s_d, self.topk_d, self.buf.mask, self.buf.perm, self.buf.stats,
                            self.packets)
        self.stats = ctx.mw_get_send_stats(self.buf.stats)
        self.N = int(self.stats["n_rows"])

    def names(self, rank: int) -> torch.Tensor:
        """Which of the N packets name `rank` (read from the packets' own headers; test plumbing
        standing in for the network)."""
        word = self.packets[: self.N, 8 * (rank >> 6): 8 * (rank >> 6) + 8].contiguous().view(torch.int64)[:, 0]
        return ((word >> (rank & 63)) & 1).bool()


def unpack_packets(ctx, regions, capacity):
    table = B.packets_table(regions, [r.shape[0] if r.numel() else 0 for r in regions], H.DEV)
    buf = B.RecvBuffers(ctx, capacity)
    ctx.mw_unpack_packets(table, len(regions), buf.out_rows, buf.out_scales, capacity, buf.out_src_peer,
                          buf.out_src_token, buf.expert_offsets, buf.stats)
    st = ctx.mw_get_recv_stats(buf.stats)
    q = min(int(st["n_out_rows"]), capacity)
    out = (H.host(buf.out_rows)[:q], None if buf.out_scales is None else H.host(buf.out_scales)[:q],
           H.host(buf.out_src_peer)[:q], H.host(buf.out_src_token)[:q], H.host(buf.expert_offsets))
    return out, st


def same(got, want, what):
    H.assert_same_bytes(got[4], want[4], what + " expert_offsets")
    H.assert_same_bytes(got[2], want[2], what + " out_src_peer")
    H.assert_same_bytes(got[3], want[3], what + " out_src_token")
    H.assert_same_bytes(got[0], want[0], what + " out_rows")
    if want[1] is not None:
        H.assert_same_bytes(got[1], want[1], what + " out_scales")


def run_packets(w, seed, my_rank, lazy=False, check_senders=None, complete_too=False, edit=None):
    _say("packets", w.name, "seed", seed, "my_rank", my_rank, "T", w.n_tokens, "H", w.hidden, w.row_format)
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, my_rank)
    topks = W.topk_ids_many(w, seed, range(w.n_ranks))
    x_dev = s_dev = None
    if lazy:
        xdt = torch.uint8 if w.row_format == "fp8" else torch.int16
        x_dev = torch.zeros((w.n_tokens, w.hidden), dtype=xdt, device=H.DEV)
        if w.row_format == "fp8":
            s_dev = torch.zeros((w.n_tokens, w.hidden // 128), dtype=torch.float32, device=H.DEV)
    gen = torch.Generator(device="cpu"); gen.manual_seed(seed)
    toks, kept, complete, shuffled, shuffled_oracle = [], [], [], [], []
    for p in range(w.n_ranks):
        tk = topks[p]
        if edit is not None:
            edit(p, tk)
        if lazy:
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
            g = GpuPackets(ctx, tk, x, sc, x_dev=x_dev, scales_dev=s_dev)
        else:
            x, sc = W.payload_rows(w, seed, p)
            g = GpuPackets(ctx, tk, x, sc)
        toks.append((tk, x, sc))
        if check_senders is None or p in check_senders:
            mask, perm, _, st = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
            want = ref.pack_packets(x, sc, tk, mask, perm)
            assert g.N == len(perm)
            H.assert_same_bytes(H.host(g.packets)[: g.N], want, "packets of peer %d" % p)
        mine = g.packets[: g.N][g.names(my_rank)].clone()
        kept.append(mine)
        if complete_too:
            complete.append(g.packets[: g.N].clone())
            order = torch.randperm(mine.shape[0], generator=gen)
            shuffled.append(mine[order.to(H.DEV)].clone())
            # the oracle parses its own packets, put into the same order
            o_mine = ref.deliver_packets(H.oracle_packets(w, tk, x, sc), my_rank)
            assert len(o_mine) == mine.shape[0]
            shuffled_oracle.append(o_mine[order.numpy()])
        del g
    m_rows = sum(int(k.shape[0]) for k in kept)
    cap = max(1, m_rows * min(w.top_k, w.experts_per_rank))
    want = ref.dispatch_plain(toks, e2r, my_rank, cap)
    got, st = unpack_packets(ctx, kept, cap)
    assert int(st["error_flags"]) == 0, hex(int(st["error_flags"]))
    same(got, want, "packets vs plain definition")
    assert int(st["n_recv_rows"]) == m_rows == int(st["n_rows_seen"])
    if complete_too:
        got, st = unpack_packets(ctx, complete, cap)
        assert int(st["error_flags"]) == 0 and int(st["n_recv_rows"]) == m_rows
        same(got, want, "complete sender buffers")
        got, st = unpack_packets(ctx, shuffled, cap)
        assert int(st["error_flags"]) == 0
        same(got, want, "packets in any order")
        xrb = 2 * w.hidden if w.row_format == "bf16" else w.hidden
        o2 = ref.unpack_packets(shuffled_oracle, w.top_k, e2r, my_rank, xrb, w.row_bytes - xrb, cap)
        same(got, o2, "vs the oracle's packet parser")
    _say("  packets received", m_rows, "output rows", int(st["n_out_rows"]))
    ctx.close()


@pytest.mark.parametrize("seed", [W.BASE_SEED, 1])
@pytest.mark.parametrize("my_rank", [0, 5])
def test_c0_tiny(seed, my_rank):
    run_packets(W.C0, seed, my_rank, complete_too=True)


@pytest.mark.parametrize("seed", [1, 2])
def test_c1_shape_reduced(seed):
    run_packets(W.scaled(W.C1, n_tokens=333, hidden=1024), seed, 37, complete_too=(seed == 1))


def test_c2_shape_reduced_fp8():
    run_packets(W.scaled(W.C2, n_tokens=333, hidden=1024), 1, 0, complete_too=True)


def test_c3_shape_reduced_wide_bitmaps():
    w = W.scaled(W.C3, n_tokens=200, hidden=512)
    run_packets(w, 1, W.zipf_hottest_rank(w, 1), check_senders=(0, 100, 255), complete_too=True)
    run_packets(w, 1, 200, check_senders=(3,))


def test_full_width_rows_duplicates_and_padding():
    def edit(p, tk):
        tk[p % 3::3, 1] = tk[p % 3::3, 0]
        tk[1::5, 0] = -1
        tk[7] = -1
    run_packets(W.DispatchWorkload("wide_bf16", 11, 8, 16, 2, 257, 7168, "bf16", "uniform"), 1, 3,
                complete_too=True, edit=edit)
    run_packets(W.DispatchWorkload("wide_fp8", 12, 8, 16, 2, 129, 7168, "fp8", "uniform"), 1, 6, edit=edit)
    # more ids than one 128-byte header holds: two header lines
    run_packets(W.DispatchWorkload("k24", 13, 16, 64, 24, 70, 256, "bf16", "uniform"), 2, 9, complete_too=True)


def test_more_than_eight_local_experts_per_row():
    run_packets(W.DispatchWorkload("dense20", 91, 2, 40, 24, 100, 256, "bf16", "uniform"), 1, 1, complete_too=True)
    run_packets(W.DispatchWorkload("k64", 92, 4, 128, 64, 60, 128, "bf16", "uniform"), 2, 3)


def test_c1_full_size():
    run_packets(W.C1, W.BASE_SEED, 0, lazy=True, check_senders=(7, 63))


def test_empty_regions_and_bad_headers():
    w = W.DispatchWorkload("small", 31, 8, 16, 2, 128, 256, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, 0)
    hb = B.mw_packet_header_bytes(w.top_k)
    assert hb == 128 == ref.packet_header_bytes(w.top_k)
    empty = torch.zeros((0, hb + w.row_bytes), dtype=torch.uint8, device=H.DEV)
    got, st = unpack_packets(ctx, [empty, empty], 4)
    assert int(st["n_out_rows"]) == 0 and int(st["error_flags"]) == 0 and got[4].tolist() == [0, 0, 0]
    tk = W.topk_ids(w, 1, 0)
    x, _ = W.payload_rows(w, 1, 0)
    g = GpuPackets(ctx, tk, x, None)
    mine = g.packets[: g.N][g.names(0)].clone()
    want = ref.dispatch_plain([(tk, x, None)], e2r, 0, 1000)
    got, st = unpack_packets(ctx, [mine], 1000)
    same(got, want, "one peer")
    # a header that says K = 3: that packet is left out and flagged; the others are delivered
    o_mine = ref.deliver_packets(H.oracle_packets(w, tk, x, None), 0)
    H.assert_same_bytes(H.host(mine), o_mine, "packets naming rank 0")
    victim = 4
    bad_o = o_mine.copy()
    bad_o[victim, 36] = 3
    bad = H.dev(bad_o)
    tok = int(bad_o[victim, 32:36].view(np.int32)[0])
    tk2 = tk.copy(); tk2[tok] = -1
    want2 = ref.dispatch_plain([(tk2, x, None)], e2r, 0, 1000)
    got, st = unpack_packets(ctx, [bad], 1000)
    assert int(st["error_flags"]) == B.MW_FLAG_BAD_DESC
    same(got, want2, "bad header left out")
    with pytest.raises(ref.OracleError):
        ref.unpack_packets([bad_o], w.top_k, e2r, 0, w.row_bytes, 0, 1000)
    # the flag does not stick
    got, st = unpack_packets(ctx, [mine], 1000)
    assert int(st["error_flags"]) == 0
    # the descriptor path on the same context still works after the packet path
    gs = H.GpuSend(ctx, tk, x, None)
    gu = H.GpuUnpack(ctx, [H.shrink(gs.deliver(0))], 1000)
    H.check_unpack(gu, want, "descriptor path after packets")
    ctx.close()


# ------------------------------------------------------------------ relay of packets
def _relay_ctx(w, my_rank, max_hops):
    return B.Context(w.n_ranks, w.n_experts, w.top_k, my_rank, w.hidden, H.fmt_code(w), max(w.n_tokens, 1),
                     w.n_ranks * w.n_tokens, W.expert_to_rank(w), device=H.DEV, max_hops=max_hops)


def gpu_relay_packets(ctx, packets, n_rows, next_hop, n_hops, capacity):
    ctx.mw_set_forwarding(next_hop, n_hops)
    pb = packets.shape[1]
    kids = [torch.zeros((max(capacity, 1), pb), dtype=torch.uint8, device=H.DEV) for _ in range(n_hops)]
    table = torch.tensor([k.data_ptr() for k in kids], dtype=torch.int64, device=H.DEV)
    rec = B.packets_table([packets], [n_rows], H.DEV)
    stats = torch.zeros(B.RELAY_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    ctx.mw_relay_packets(rec, table, capacity, stats)
    st = ctx.mw_get_relay_stats(stats)
    return kids, st


@pytest.mark.parametrize("which", ["c0", "c1_reduced", "c3_reduced", "fp8", "ep96", "ep200"])
def test_relay_packets_children_and_accounting(which):
    import dataclasses
    w = {"c0": W.C0, "c1_reduced": W.scaled(W.C1, n_tokens=333, hidden=1024),
         "c3_reduced": W.scaled(W.C3, n_tokens=200, hidden=512),
         # bitmaps of two words and of four with the last partly used (the index reads only the words that can name a rank)
         "ep96": dataclasses.replace(W.C3, name="ep96", n_ranks=96, n_experts=192, n_tokens=300, hidden=512),
         "ep200": dataclasses.replace(W.C3, name="ep200", n_ranks=200, n_experts=200, n_tokens=1100, hidden=256),
         "fp8": W.scaled(W.C2, n_tokens=150, hidden=1024)}[which]
    _say("relay packets", w.name)
    n_per = 8
    me = 9 % w.n_ranks
    next_hop = np.array([(r % n_per) if r // n_per == me // n_per else n_per + (r // n_per) -
                         (1 if r // n_per > me // n_per else 0) for r in range(w.n_ranks)], dtype=np.int32)
    n_hops = int(next_hop.max()) + 1
    ctx = _relay_ctx(w, me, n_hops)
    tk = W.topk_ids(w, 3, me)
    x, sc = W.payload_rows(w, 3, me)
    g = GpuPackets(ctx, tk, x, sc)
    kids, st = gpu_relay_packets(ctx, g.packets, g.N, next_hop, n_hops, w.n_tokens)
    parent = H.oracle_packets(w, tk, x, sc)
    H.assert_same_bytes(H.host(g.packets)[: g.N], parent, "packets before the relay")
    pb = parent.shape[1]
    total = 0
    for h in range(n_hops):
        want, copies, dests = ref.relay_packets_child(parent, next_hop, n_hops, h)
        n = int(st["rows_per_hop"][h])
        assert n == len(want) == int(st["groups_per_hop"][h])
        H.assert_same_bytes(H.host(kids[h])[:n], want, "child %d packets" % h)
        total += n
    assert int(st["error_flags"]) == 0
    assert (int(st["n_rows_in"]), int(st["n_groups_in"])) == (g.N, g.N)
    assert int(st["forward_bytes"]) == copies * pb == total * pb
    assert int(st["unicast_bytes"]) == dests * pb
    ctx.close()


def test_delivery_through_relayed_packets_equals_direct_delivery():
    """Two servers of four devices: every sender's packets go through a server-level relay and a
    device-level relay on the GPU; what reaches my_rank is unpacked and compared with the plain
    definition of the dispatch."""
    w = W.DispatchWorkload("two_level", 81, 8, 24, 4, 90, 256, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    my_rank = 6
    ctx = _relay_ctx(w, my_rank, 4)
    to_server = np.array([r // 4 for r in range(8)], dtype=np.int32)
    to_device = np.array([r % 4 for r in range(8)], dtype=np.int32)
    toks, regions = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, 5, p)
        x, _ = W.payload_rows(w, 5, p)
        toks.append((tk, x, None))
        g = GpuPackets(ctx, tk, x, None)
        kids, st = gpu_relay_packets(ctx, g.packets, g.N, to_server, 2, w.n_tokens)
        n1 = int(st["rows_per_hop"][my_rank // 4])
        at_server = kids[my_rank // 4][:max(n1, 1)].clone()
        kids2, st2 = gpu_relay_packets(ctx, at_server, n1, to_device, 4, w.n_tokens)
        n2 = int(st2["rows_per_hop"][my_rank % 4])
        assert int(st["error_flags"]) == 0 and int(st2["error_flags"]) == 0
        mine = kids2[my_rank % 4][:n2].clone()
        # down to a plain write: only my_rank is left in every bitmap
        words = H.host(mine)[:, :32].copy().view(np.uint64)
        assert np.all(words[:, 0] == np.uint64(1 << my_rank)) and not words[:, 1:].any()
        regions.append(mine)
    cap = 10 ** 4
    want = ref.dispatch_plain(toks, e2r, my_rank, cap)
    got, st = unpack_packets(ctx, regions, cap)
    assert int(st["error_flags"]) == 0
    same(got, want, "through two relay levels")
    ctx.close()


def test_relay_packets_capacity_and_bad_headers():
    w = W.DispatchWorkload("small", 31, 8, 16, 2, 128, 256, "bf16", "uniform")
    ctx = _relay_ctx(w, 0, 2)
    tk = W.topk_ids(w, 1, 0)
    x, _ = W.payload_rows(w, 1, 0)
    g = GpuPackets(ctx, tk, x, None)
    next_hop = np.array([0, 0, 0, 0, 1, 1, 1, 1], dtype=np.int32)
    parent = H.oracle_packets(w, tk, x, None)
    want0, _, _ = ref.relay_packets_child(parent, next_hop, 2, 0)
    cap = len(want0) // 2
    kids, st = gpu_relay_packets(ctx, g.packets, g.N, next_hop, 2, cap)
    assert int(st["error_flags"]) == B.MW_FLAG_OUT_CAPACITY
    assert int(st["rows_per_hop"][0]) == cap
    H.assert_same_bytes(H.host(kids[0])[:cap], want0[:cap], "packets below the capacity are still exact")
    # a header with another id count: the packet is forwarded nowhere
    bad = g.packets.clone()
    bad[3, 36] = 7
    kids, st = gpu_relay_packets(ctx, bad, g.N, next_hop, 2, w.n_tokens)
    assert int(st["error_flags"]) == B.MW_FLAG_BAD_DESC and int(st["n_rows_in"]) == g.N - 1
    rest = np.delete(parent, 3, axis=0)
    for h in range(2):
        want, _, _ = ref.relay_packets_child(rest, next_hop, 2, h)
        n = int(st["rows_per_hop"][h])
        H.assert_same_bytes(H.host(kids[h])[:n], want, "child %d without the bad packet" % h)
    kids, st = gpu_relay_packets(ctx, g.packets, g.N, next_hop, 2, w.n_tokens)
    assert int(st["error_flags"]) == 0                    # flags do not stick
    ctx.close()


@pytest.mark.parametrize("which", ["c1_reduced", "long_packets", "fp8"])
def test_relay_packets_stream_index_of_the_next_buffer_rides_with_the_copy(which):
    """mw_relay_packets_index + mw_relay_packets_copy_index_next + mw_relay_packets_copy over a
    stream of packet buffers on two contexts with different forwarding tables: every step's
    children and statistics against the oracle; one buffer is short and one is empty."""
    w = {"c1_reduced": W.scaled(W.C1, n_tokens=300, hidden=1024),
         "long_packets": W.scaled(W.C1, n_tokens=120, hidden=7168),      # 904 chunks: three 320-lane workgroups per packet
         "fp8": W.scaled(W.C2, n_tokens=200, hidden=1024)}[which]
    _say("relay packets stream", w.name)
    rng = np.random.default_rng(6)
    tables = [(rng.integers(0, 7, size=w.n_ranks).astype(np.int32), 7),
              (rng.integers(0, 20, size=w.n_ranks).astype(np.int32), 20)]
    ctxs = [_relay_ctx(w, 0, 64), _relay_ctx(w, 0, 64)]
    for c, (nh, n) in zip(ctxs, tables):
        c.mw_set_forwarding(nh, n)
    steps = []
    for i, T in enumerate([w.n_tokens, 50, 0, w.n_tokens]):
        tk = W.topk_ids(w, 60 + i, i)[:T].copy()
        x, sc = W.payload_rows(w, 60 + i, i)
        x, sc = x[:T].copy(), (None if sc is None else sc[:T].copy())
        g = GpuPackets(ctxs[0], tk, x, sc)
        n = tables[i % 2][1]
        pb = g.packets.shape[1]
        kids = [torch.zeros((w.n_tokens, pb), dtype=torch.uint8, device=H.DEV) for _ in range(n)]
        steps.append(dict(tk=tk, x=x, sc=sc, g=g, kids=kids, rec=B.packets_table([g.packets], [g.N], H.DEV),
                          table=torch.tensor([k.data_ptr() for k in kids], dtype=torch.int64, device=H.DEV),
                          stats=torch.zeros(B.RELAY_STATS_BYTES, dtype=torch.uint8, device=H.DEV)))
    ctxs[0].mw_relay_packets_index(steps[0]["rec"], w.n_tokens, steps[0]["stats"])
    for i, st in enumerate(steps):
        cur = ctxs[i % 2]
        if i + 1 < len(steps):
            nx = steps[i + 1]
            cur.mw_relay_packets_copy_index_next(st["rec"], st["table"], st["stats"], ctxs[(i + 1) % 2], nx["rec"],
                                                 w.n_tokens, nx["stats"])
        else:
            cur.mw_relay_packets_copy(st["rec"], st["table"], st["stats"])
    torch.cuda.synchronize()
    for i, st in enumerate(steps):
        nh, n = tables[i % 2]
        got = ctxs[i % 2].mw_get_relay_stats(st["stats"])
        parent = H.oracle_packets(w, st["tk"], st["x"], st["sc"])
        pb, total, copies, dests = st["g"].packets.shape[1], 0, 0, 0
        for h in range(n):
            want, copies, dests = ref.relay_packets_child(parent, nh, n, h)
            k = int(got["rows_per_hop"][h])
            assert k == len(want) == int(got["groups_per_hop"][h])
            H.assert_same_bytes(H.host(st["kids"][h])[:k], want, "step %d child %d packets" % (i, h))
            total += k
        assert int(got["error_flags"]) == 0 and int(got["n_rows_in"]) == st["g"].N
        assert int(got["forward_bytes"]) == copies * pb == total * pb and int(got["unicast_bytes"]) == dests * pb
    with pytest.raises(B.MwError) as ei:
        ctxs[0].mw_relay_packets_copy_index_next(steps[0]["rec"], steps[0]["table"], steps[0]["stats"], ctxs[0],
                                                 steps[1]["rec"], w.n_tokens, steps[1]["stats"])
    assert ei.value.status == B.MW_ERR_INVALID_ARG
    for c in ctxs:
        c.close()
