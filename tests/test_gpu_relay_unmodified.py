"""GPU parity of the two context options of Section 4.1's last paragraph of "Replication and
forwarding": relays that forward the metadata as it came (MW_OPT_RELAY_KEEP_METADATA) and end
nodes that drop repeated rows (MW_OPT_RECV_DEDUP), in the descriptor-table and the packets form,
against the CPU oracle on the same seeded inputs.  Bit-exact."""
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


def _ctx(w, my_rank, max_hops, max_tokens, options):
    ctx = B.Context(w.n_ranks, w.n_experts, w.top_k, my_rank, w.hidden, H.fmt_code(w), max_tokens,
                    w.n_ranks * max_tokens, W.expert_to_rank(w), device=H.DEV, max_hops=max_hops)
    ctx.mw_ctx_set_options(options)
    return ctx


def _relay(ctx, rec, next_hop, n_hops, capacity):
    ctx.mw_set_forwarding(next_hop, n_hops)
    ch = B.RelayChildren(ctx, n_hops, capacity)
    table = B.peers_table([rec], H.DEV)
    ctx.mw_relay(table, ch.table, capacity, ch.stats)
    st = ctx.mw_get_relay_stats(ch.stats)
    return ch, st, table


def _child_host(ch, st, h, row_bytes):
    g, n = int(st["groups_per_hop"][h]), int(st["rows_per_hop"][h])
    return (H.host(ch.desc[h]).reshape(-1).view(B.DESC_DTYPE)[:g], H.host(ch.rows[h])[:n, :row_bytes],
            H.host(ch.row_src_token[h])[:n], H.host(ch.row_topk[h])[:n])


@pytest.mark.parametrize("fmt,seed,n_hops", [("bf16", 1, 5), ("bf16", 2, 33), ("fp8", 3, 17)])
def test_children_keep_the_parents_bitmaps(fmt, seed, n_hops):
    w = W.scaled(W.C1 if fmt == "bf16" else W.C2, n_tokens=333, hidden=1024)
    _say("relay, metadata kept:", w.name, "seed", seed, "hops", n_hops)
    rng = np.random.default_rng(seed)
    next_hop = rng.integers(0, n_hops, size=w.n_ranks).astype(np.int32)
    ctx = _ctx(w, 0, 64, w.n_tokens, B.MW_OPT_RELAY_KEEP_METADATA)
    tk = W.topk_ids(w, seed, 0)
    x, sc = W.payload_rows(w, seed, 0)
    g = H.GpuSend(ctx, tk, x, sc)
    ch, st, _ = _relay(ctx, g.full_record(), next_hop, n_hops, w.n_tokens)
    parent = H.oracle_send(w, tk, x, sc)
    for h in range(n_hops):
        want = ref.relay_child(*parent, next_hop, n_hops, h, update_metadata=False)
        got = _child_host(ch, st, h, w.row_bytes)
        for a, b, what in zip(got, want, ("desc", "rows", "src_token", "row_topk")):
            H.assert_same_bytes(a.view(np.uint8), b.view(np.uint8), "child %d %s" % (h, what))
    # the copies made, hence the accounting, are those of the updating relay
    fwd, uni, rph = ref.relay_accounting(parent[0], w.row_bytes, next_hop, n_hops)
    assert int(st["error_flags"]) == 0
    assert (int(st["forward_bytes"]), int(st["unicast_bytes"])) == (fwd, uni)
    assert st["rows_per_hop"][:n_hops].tolist() == rph.tolist()
    # option off again: the updating relay
    ctx.mw_ctx_set_options(0)
    ch, st, _ = _relay(ctx, g.full_record(), next_hop, n_hops, w.n_tokens)
    for h in (0, n_hops - 1):
        want = ref.relay_child(*parent, next_hop, n_hops, h)
        got = _child_host(ch, st, h, w.row_bytes)
        H.assert_same_bytes(got[0].view(np.uint8), want[0].view(np.uint8), "updated child %d desc" % h)
    with pytest.raises(B.MwError):
        ctx.mw_ctx_set_options(0x80)                  # no such option
    ctx.close()


def _gpu_concat(recs, row_stride, top_k):
    """Several received buffers of one source as one region on the device: descriptors one after
    the other with their row ranges rebased (plumbing standing in for the network: what lands in
    a peer's receive region over more than one path)."""
    descs, rows, src, rtk, off = [], [], [], [], 0
    for r in recs:
        g, n = r["n_desc"], r["n_rows"]
        d = H.host(r["desc"]).reshape(-1).view(B.DESC_DTYPE)[:g].copy()
        d["row_offset"] += np.uint32(off)
        off += n
        descs.append(d)
        rows.append(r["rows"][:n]); src.append(r["row_src_token"][:n]); rtk.append(r["row_topk"][:n])
    d = np.concatenate(descs) if descs else np.zeros(0, dtype=B.DESC_DTYPE)
    if len(d) == 0:
        return dict(desc=torch.zeros((1, B.DESC_BYTES), dtype=torch.uint8, device=H.DEV),
                    rows=torch.zeros((1, row_stride), dtype=torch.uint8, device=H.DEV),
                    row_src_token=torch.zeros(1, dtype=torch.int32, device=H.DEV),
                    row_topk=torch.zeros((1, top_k), dtype=torch.int32, device=H.DEV), n_desc=0, n_rows=0)
    return dict(desc=H.dev(d.view(np.uint8).reshape(-1, B.DESC_BYTES)), rows=torch.cat(rows).contiguous(),
                row_src_token=torch.cat(src).contiguous(), row_topk=torch.cat(rtk).contiguous(),
                n_desc=len(d), n_rows=off)


def _oracle_concat(bufs, row_bytes, top_k):
    descs, rows, src, rtk, off = [], [], [], [], 0
    for d, r, s, t in bufs:
        d = d.copy()
        d["row_offset"] += np.uint32(off)
        off += len(r)
        descs.append(d); rows.append(r); src.append(s); rtk.append(t)
    if not descs:
        return (np.zeros(0, dtype=ref.DESC), np.zeros((0, row_bytes), np.uint8), np.zeros(0, np.int32),
                np.zeros((0, top_k), np.int32))
    return (np.concatenate(descs), np.concatenate(rows), np.concatenate(src), np.concatenate(rtk))


@pytest.mark.parametrize("fmt,seed", [("bf16", 1), ("bf16", 2), ("fp8", 3)])
def test_delivery_over_relays_that_keep_the_metadata_with_dedup_at_the_end_nodes(fmt, seed):
    """A loop-free deployment of the two options, everything on the GPU: every source reaches some
    ranks directly and the others through two relay ranks; the relays forward once, to every rank
    their (unmodified) bitmaps name; end nodes never forward.  A destination then holds the same
    (source, token) row once per path.  mw_unpack with MW_OPT_RECV_DEDUP is compared with the
    oracle's de-duplicating receive side on the oracle's own regions and with the plain
    definition of the dispatch; without the option the repeats are reported as an input error."""
    rng = np.random.default_rng(seed)
    hidden = 512 if fmt == "bf16" else 1024
    w = W.DispatchWorkload("keep", 36 + seed, 10, 20, 3, 150, hidden, fmt, "uniform")
    _say("relays keep metadata, end nodes de-duplicate:", fmt, "seed", seed)
    e2r = W.expert_to_rank(w)
    R, T = w.n_ranks, w.n_tokens
    relays = [2, 7]
    cap_rows = 3 * T                                   # a region holds a row at most once per path
    rctx = _ctx(w, 0, 16, cap_rows, B.MW_OPT_RELAY_KEEP_METADATA)
    ident = np.arange(R, dtype=np.int32)
    dests = (0, 2, 5, 9)
    toks = []
    gpu_regions = {d: [] for d in dests}
    ora_regions = {d: [] for d in dests}
    keep = []
    for s in range(R):
        tk = W.topk_ids(w, seed, s)
        x, sc = W.payload_rows(w, seed, s)
        toks.append((tk, x, sc))
        via = rng.integers(0, 1 + len(relays), size=R).astype(np.int32)
        via[s] = 0
        for rl in relays:
            if rl == s:
                via[rl] = 0
        # ---- GPU
        g = H.GpuSend(rctx, tk, x, sc)
        ch, st, _ = _relay(rctx, g.full_record(), via, 1 + len(relays), cap_rows)
        assert int(st["error_flags"]) == 0
        keep += [g, ch]
        arrivals = {d: [] for d in dests}
        for d in dests:
            if via[d] == 0:
                arrivals[d].append(ch.record(0, int(st["groups_per_hop"][0]), int(st["rows_per_hop"][0])))
        for j, rl in enumerate(relays):
            ng, nr = int(st["groups_per_hop"][1 + j]), int(st["rows_per_hop"][1 + j])
            if ng == 0:
                continue
            to_relay = ch.record(1 + j, ng, nr)
            ch2, st2, _ = _relay(rctx, to_relay, ident, R, cap_rows)
            assert int(st2["error_flags"]) == 0
            keep.append(ch2)
            for d in dests:
                if d != s and d != rl:
                    arrivals[d].append(ch2.record(d, int(st2["groups_per_hop"][d]), int(st2["rows_per_hop"][d])))
            if rl in dests and via[rl] == 1 + j:
                arrivals[rl].append(to_relay)
        for d in dests:
            gpu_regions[d].append(_gpu_concat(arrivals[d], rctx.row_stride, w.top_k))
        # ---- the oracle, on its own buffers
        parent = H.oracle_send(w, tk, x, sc)
        o_arr = {d: [] for d in dests}
        direct = ref.relay_child(*parent, via, 1 + len(relays), 0, update_metadata=False)
        for d in dests:
            if via[d] == 0:
                o_arr[d].append(direct)
        for j, rl in enumerate(relays):
            to_relay = ref.relay_child(*parent, via, 1 + len(relays), 1 + j, update_metadata=False)
            if len(to_relay[0]) == 0:
                continue
            for d in dests:
                if d != s and d != rl:
                    o_arr[d].append(ref.relay_child(*to_relay, ident, R, d, update_metadata=False))
            if rl in dests and via[rl] == 1 + j:
                o_arr[rl].append(to_relay)
        for d in dests:
            ora_regions[d].append(_oracle_concat(o_arr[d], w.row_bytes, w.top_k))
    n_dropped = 0
    for d in dests:
        cap = 3 * sum(r["n_rows"] for r in gpu_regions[d]) + 4
        xrb = 2 * w.hidden if fmt == "bf16" else w.hidden
        want = ref.unpack_dedup(ora_regions[d], w.top_k, e2r, d, xrb, w.row_bytes - xrb, cap)
        plain = ref.dispatch_plain(toks, e2r, d, cap)
        taken, dropped = want[5]
        for a, b in zip(want[:5], plain[:5]):
            assert (a is None and b is None) or a.tobytes() == b.tobytes()
        ctx = _ctx(w, d, 1, cap_rows, B.MW_OPT_RECV_DEDUP)
        gu = H.GpuUnpack(ctx, gpu_regions[d], cap)
        flags = int(gu.stats["error_flags"])
        assert flags == (B.MW_FLAG_DUPLICATE_DROPPED if dropped else 0), hex(flags)
        o = gu.host_out()
        for i, what in ((4, "expert_offsets"), (2, "out_src_peer"), (3, "out_src_token"), (0, "out_rows"), (1, "out_scales")):
            if want[i] is not None:
                H.assert_same_bytes(o[i], want[i], "dest %d %s" % (d, what))
        assert int(gu.stats["n_recv_rows"]) == taken
        n_dropped += dropped
        # the same regions without the option: repeats are an input error there
        ctx.mw_ctx_set_options(0)
        gu = H.GpuUnpack(ctx, gpu_regions[d], cap)
        if dropped:
            assert int(gu.stats["error_flags"]) & B.MW_FLAG_DUP_SRC_TOKEN
        else:
            H.check_unpack(gu, plain, "no repeats, no option")
        ctx.close()
    assert n_dropped > 0
    _say("  repeats dropped over", len(dests), "destinations:", n_dropped)
    rctx.close()


def _gpu_relay_packets(ctx, packets, n_rows, next_hop, n_hops, capacity):
    ctx.mw_set_forwarding(next_hop, n_hops)
    pb = packets.shape[1]
    kids = [torch.zeros((max(capacity, 1), pb), dtype=torch.uint8, device=H.DEV) for _ in range(n_hops)]
    table = torch.tensor([k.data_ptr() for k in kids], dtype=torch.int64, device=H.DEV)
    rec = B.packets_table([packets], [n_rows], H.DEV)
    stats = torch.zeros(B.RELAY_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    ctx.mw_relay_packets(rec, table, capacity, stats)
    return kids, ctx.mw_get_relay_stats(stats)


def _gpu_packets(ctx, tk, x, sc):
    T = tk.shape[0]
    buf = B.SendBuffers(ctx, T)
    tk_d, x_d, s_d = H.dev(tk.astype(np.int32)), H.dev(x), H.dev(sc)
    packets = torch.zeros((max(T, 1), B.mw_packet_header_bytes(ctx.top_k) + ctx.row_bytes), dtype=torch.uint8,
                          device=H.DEV)
    ctx.mw_plan(tk_d, buf.mask, buf.perm, buf.desc, buf.stats)
    ctx.mw_pack_packets(x_d, s_d, tk_d, buf.mask, buf.perm, buf.stats, packets)
    return packets, int(ctx.mw_get_send_stats(buf.stats)["n_rows"])


@pytest.mark.parametrize("fmt,seed", [("bf16", 1), ("fp8", 2)])
def test_packets_relayed_with_their_headers_kept_and_de_duplicated_at_the_end_node(fmt, seed):
    """The packets' form: every child holds the kept packets byte for byte (oracle: the unmodified
    packets relay); a destination that receives a source's packets over two paths and drops the
    repeats delivers what the plain definition of the dispatch gives."""
    rng = np.random.default_rng(seed)
    w = W.DispatchWorkload("keep_pk", 46 + seed, 12, 24, 3, 140, 512 if fmt == "bf16" else 1024, fmt, "uniform")
    _say("packets relay, headers kept:", fmt, "seed", seed)
    e2r = W.expert_to_rank(w)
    R, T = w.n_ranks, w.n_tokens
    n_hops = 4
    d = 5
    rctx = _ctx(w, 0, 16, 2 * T, B.MW_OPT_RELAY_KEEP_METADATA)
    uctx = _ctx(w, d, 1, 2 * T, B.MW_OPT_RECV_DEDUP)
    toks, regions, counts = [], [], []
    total = 0
    for s in range(R):
        tk = W.topk_ids(w, seed, s)
        x, sc = W.payload_rows(w, seed, s)
        toks.append((tk, x, sc))
        next_hop = rng.integers(0, n_hops, size=R).astype(np.int32)
        packets, N = _gpu_packets(rctx, tk, x, sc)
        kids, st = _gpu_relay_packets(rctx, packets, N, next_hop, n_hops, T)
        assert int(st["error_flags"]) == 0
        parent = H.oracle_packets(w, tk, x, sc)
        for h in range(n_hops):
            want = ref.relay_packets_child(parent, next_hop, n_hops, h, update_metadata=False)
            n = int(st["rows_per_hop"][h])
            assert n == len(want)
            H.assert_same_bytes(H.host(kids[h])[:n], want, "source %d child %d packets" % (s, h))
        # two of the children reach the destination (the hop it sits behind and one other): every
        # packet that names ranks behind both arrives twice
        a, b = int(next_hop[d]), (int(next_hop[d]) + 1) % n_hops
        na, nb = int(st["rows_per_hop"][a]), int(st["rows_per_hop"][b])
        region = torch.cat([kids[a][:na], kids[b][:nb]]).contiguous()
        total += na + nb
        counts.append(na + nb)
        regions.append(region if na + nb else torch.zeros((1, packets.shape[1]), dtype=torch.uint8, device=H.DEV))
    cap = 3 * total + 4
    want = ref.dispatch_plain(toks, e2r, d, cap)
    table = B.packets_table(regions, counts, H.DEV)
    buf = B.RecvBuffers(uctx, cap)
    uctx.mw_unpack_packets(table, len(regions), buf.out_rows, buf.out_scales, cap, buf.out_src_peer,
                           buf.out_src_token, buf.expert_offsets, buf.stats)
    st = uctx.mw_get_recv_stats(buf.stats)
    assert int(st["error_flags"]) == B.MW_FLAG_DUPLICATE_DROPPED, hex(int(st["error_flags"]))
    q = int(st["n_out_rows"])
    H.assert_same_bytes(H.host(buf.expert_offsets), want[4], "expert_offsets")
    H.assert_same_bytes(H.host(buf.out_src_peer)[:q], want[2], "out_src_peer")
    H.assert_same_bytes(H.host(buf.out_src_token)[:q], want[3], "out_src_token")
    H.assert_same_bytes(H.host(buf.out_rows)[:q], want[0], "out_rows")
    if want[1] is not None:
        H.assert_same_bytes(H.host(buf.out_scales)[:q], want[1], "out_scales")
    # rows taken = tokens of all sources with an expert on d (each once)
    n_tokens_for_d = sum(len(W.tokens_for_rank(w, t[0], d)) for t in toks)
    assert int(st["n_recv_rows"]) == n_tokens_for_d
    rctx.close(); uctx.close()
