"""GPU parity on randomly drawn small configurations: rank counts, expert placements that are
not uniform (ranks with no expert, ranks with many), top-k of any size with padding and
duplicate ids, row widths that are not multiples of a wave, batch sizes around the tile sizes.
Every stage against the CPU oracle, bit-exact."""
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


def draw_config(rng):
    R = int(rng.choice([1, 2, 3, 7, 8, 16, 33, 64, 65, 100, 129, 200, 256]))
    E = int(rng.integers(1, 4 * R + 2))
    K = int(rng.choice([1, 2, 3, 4, 6, 8, 9, 12, 17]))
    T = int(rng.choice([1, 2, 63, 64, 65, 100, 255, 256, 257, 300, 513]))
    hidden = int(rng.choice([8, 24, 64, 200, 512, 1000, 1024, 2056]))       # bf16: rows of 16 .. 4112 bytes
    placement = rng.choice(["uniform", "random", "skewed"])
    if placement == "uniform":
        e2r = (np.arange(E) * R // E).astype(np.int32)
    elif placement == "random":
        e2r = rng.integers(0, R, size=E).astype(np.int32)
    else:                                                                     # most experts on few ranks
        hot = rng.integers(0, R, size=max(1, R // 8))
        e2r = np.where(rng.random(E) < 0.7, rng.choice(hot, size=E), rng.integers(0, R, size=E)).astype(np.int32)
    return R, E, K, T, hidden, e2r


def draw_tokens(rng, T, K, E, hidden):
    tk = rng.integers(0, E, size=(T, K)).astype(np.int32)                     # duplicates happen by themselves
    tk[rng.random((T, K)) < 0.2] = -1                                         # padding
    if T > 3:
        tk[rng.integers(0, T, size=max(1, T // 10))] = -1                     # tokens that go nowhere
    x = rng.integers(0, 1 << 16, size=(T, hidden), dtype=np.uint16)           # any bit patterns: bytes only
    return tk, x


@pytest.mark.parametrize("case", range(24))
def test_random_configuration(case):
    rng = np.random.default_rng(1000 + case)
    R, E, K, T, hidden, e2r = draw_config(rng)
    _run_configuration(rng, case, R, E, K, T, hidden, e2r)


@pytest.mark.parametrize("hidden", [5120, 5128, 5184, 8200])
def test_long_rows_through_every_entry_point(hidden):
    """Rows of 640, 641, 648 and 1025 chunks (the launch shape of the row movers changes between
    them) through plan, pack, delivery, unpack, packets and the way back."""
    rng = np.random.default_rng(3000 + hidden)
    R, E, K, T, _, e2r = draw_config(rng)
    _run_configuration(rng, hidden, R, E, K, min(T, 100), hidden, e2r)


def _run_configuration(rng, case, R, E, K, T, hidden, e2r):
    counts = np.bincount(e2r, minlength=R)
    my_rank = int(rng.choice([int(np.argmax(counts)), int(rng.integers(0, R))]))
    L = int(counts[my_rank])
    rb = 2 * hidden
    _say("case", case, "R", R, "E", E, "K", K, "T", T, "hidden", hidden, "my_rank", my_rank, "local experts", L)
    n_peers = min(R, int(rng.choice([1, 2, 5, R])))
    ctx = B.Context(R, E, K, my_rank, hidden, B.MW_ROW_BF16, T, n_peers * T, e2r, device=H.DEV)
    toks, recs, bufs, pk_regions = [], [], [], []
    hb = B.mw_packet_header_bytes(K)
    for p in range(n_peers):
        tk, x = draw_tokens(rng, T, K, E, hidden)
        toks.append((tk, x, None))
        g = H.GpuSend(ctx, tk, x, None, fused=(T <= B.MW_FUSED_MAX_TOKENS and p % 2 == 1))
        mask, perm, desc, st = ref.plan(tk, e2r, R, rb)
        gm, gperm, gdesc = g.host_plan()
        H.assert_same_bytes(gm, mask, "mask")
        H.assert_same_bytes(gperm, perm, "perm")
        H.assert_same_bytes(gdesc.view(np.uint8), desc.view(np.uint8), "desc")
        for f in ("n_rows", "n_groups", "multicast_bytes", "unicast_bytes", "error_flags"):
            assert int(g.stats[f]) == int(st[f]), f
        H.assert_same_bytes(g.stats["rows_per_dest"], st["rows_per_dest"], "rows_per_dest")
        packed, src, rtk = ref.pack(x, None, tk, perm)
        gp, gs, gt = g.host_pack()
        H.assert_same_bytes(gp, packed, "packed rows")
        H.assert_same_bytes(gs, src, "row_src_token")
        H.assert_same_bytes(gt, rtk, "row_topk")
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
        rec = H.shrink(g.deliver(my_rank))
        for a, b, name in zip(H.record_host(rec), bufs[-1], ("desc", "rows", "src_token", "row_topk")):
            H.assert_same_bytes(a.view(np.uint8) if name == "desc" else a, b.view(np.uint8) if name == "desc" else b,
                                "deliver " + name)
        recs.append(rec)
        # the same sender's traffic as packets
        pk = torch.zeros((max(T, 1), hb + rb), dtype=torch.uint8, device=H.DEV)
        ctx.mw_pack_packets(g.x_d, None, g.topk_d, g.buf.mask, g.buf.perm, g.buf.stats, pk)
        want_pk = ref.pack_packets(x, None, tk, mask, perm)
        H.assert_same_bytes(H.host(pk)[: len(perm)], want_pk, "packets")
        pk_regions.append(H.dev(ref.deliver_packets(want_pk, my_rank)) if len(want_pk) else pk[:0])
    m_rows = sum(r["n_rows"] for r in recs)
    cap = max(1, m_rows * max(1, min(K, L)))
    plain = ref.dispatch_plain(toks, e2r, my_rank, cap)
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, plain, "unpack vs plain definition")
    assert int(gu.stats["n_recv_rows"]) == m_rows
    # packets give the same
    table = B.packets_table(pk_regions, [int(r.shape[0]) for r in pk_regions], H.DEV)
    buf = B.RecvBuffers(ctx, cap)
    ctx.mw_unpack_packets(table, n_peers, buf.out_rows, buf.out_scales, cap, buf.out_src_peer, buf.out_src_token,
                          buf.expert_offsets, buf.stats)
    st = ctx.mw_get_recv_stats(buf.stats)
    q = int(st["n_out_rows"])
    assert int(st["error_flags"]) == 0 and q == gu.Q
    H.assert_same_bytes(H.host(buf.out_rows)[:q], plain[0], "packets out_rows")
    H.assert_same_bytes(H.host(buf.out_src_token)[:q], plain[3], "packets out_src_token")
    H.assert_same_bytes(H.host(buf.expert_offsets), plain[4], "packets expert_offsets")
    # the way back on the index the packet unpack left
    if q > 0 and m_rows > 0:
        y_bits = W.f32_to_bf16_bits(rng.standard_normal((q, hidden)).astype(np.float32))
        y_dev = torch.zeros((cap, hidden), dtype=torch.int16, device=H.DEV)
        y_dev[:q] = H.dev(y_bits)
        ret = torch.zeros((m_rows, hidden), dtype=torch.int16, device=H.DEV)
        ctx.mw_combine_gather(n_peers, y_dev, cap, ret, m_rows)
        torch.cuda.synchronize()
        want = np.concatenate(ref.combine_gather(bufs, K, e2r, my_rank, y_bits, plain[2], plain[3], plain[4]))
        H.assert_same_bytes(H.host(ret).view(np.uint16), want, "returned rows")
    ctx.close()


@pytest.mark.parametrize("case", range(10))
def test_random_configuration_fp8_and_relays(case):
    """fp8 rows (codes + scales), quantise-in-pack, and the relay step in both forms with a
    randomly drawn forwarding table."""
    rng = np.random.default_rng(2000 + case)
    R = int(rng.choice([2, 5, 8, 40, 64, 70, 130, 256]))
    E = int(rng.integers(R, 3 * R + 1))
    K = int(rng.choice([1, 2, 4, 8, 10]))
    T = int(rng.choice([1, 60, 64, 129, 256, 300]))
    hidden = int(rng.choice([512, 1024, 1536]))
    e2r = rng.integers(0, R, size=E).astype(np.int32)
    me = int(rng.integers(0, R))
    n_hops = int(rng.integers(1, min(R, 16) + 1))
    next_hop = rng.integers(0, n_hops, size=R).astype(np.int32)
    _say("case", case, "R", R, "E", E, "K", K, "T", T, "hidden", hidden, "hops", n_hops)
    ctx = B.Context(R, E, K, me, hidden, B.MW_ROW_FP8_E4M3_BLOCK128, T, R * T, e2r, device=H.DEV, max_hops=n_hops)
    rb = hidden + 4 * (hidden // 128)
    tk = rng.integers(0, E, size=(T, K)).astype(np.int32)
    tk[rng.random((T, K)) < 0.15] = -1
    xf = (rng.standard_normal((T, hidden)) * rng.choice([1e-3, 1.0, 300.0], size=(T, 1))).astype(np.float32)
    x_bits = W.f32_to_bf16_bits(xf)
    codes, scales = ref.quantize_rows(x_bits)
    # quantise-in-pack against quantise, then pack
    tk_d = H.dev(tk)
    sb = B.SendBuffers(ctx, T)
    ctx.mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
    ctx.mw_pack_quantize(H.dev(x_bits), tk_d, sb.perm, sb.stats, sb.packed, sb.row_src_token, sb.row_topk)
    st = ctx.mw_get_send_stats(sb.stats)
    N, G = int(st["n_rows"]), int(st["n_groups"])
    mask, perm, desc, ost = ref.plan(tk, e2r, R, rb)
    packed, src, rtk = ref.pack(codes, scales, tk, perm)
    assert N == len(perm) and G == len(desc)
    H.assert_same_bytes(H.host(sb.packed)[:N], packed, "quantised packed rows")
    # relay, descriptor form
    ctx.mw_set_forwarding(next_hop, n_hops)
    ch = B.RelayChildren(ctx, n_hops, max(T, 1))
    rec = dict(desc=sb.desc, rows=sb.packed, row_src_token=sb.row_src_token, row_topk=sb.row_topk, n_desc=G, n_rows=N)
    ctx.mw_relay(B.peers_table([rec], H.DEV), ch.table, max(T, 1), ch.stats)
    rst = ctx.mw_get_relay_stats(ch.stats)
    assert int(rst["error_flags"]) == 0
    for h in range(n_hops):
        d2, r2, s2, t2 = ref.relay_child(desc, packed, src, rtk, next_hop, n_hops, h)
        g, n = int(rst["groups_per_hop"][h]), int(rst["rows_per_hop"][h])
        assert (g, n) == (len(d2), len(r2))
        H.assert_same_bytes(H.host(ch.desc[h]).reshape(-1).view(B.DESC_DTYPE)[:g].view(np.uint8), d2.view(np.uint8),
                            "child %d desc" % h)
        H.assert_same_bytes(H.host(ch.rows[h])[:n], r2, "child %d rows" % h)
        H.assert_same_bytes(H.host(ch.row_src_token[h])[:n], s2, "child %d src_token" % h)
    fwd, uni, rph = ref.relay_accounting(desc, rb, next_hop, n_hops)
    assert (int(rst["forward_bytes"]), int(rst["unicast_bytes"])) == (fwd, uni)
    # relay, packet form
    hb = B.mw_packet_header_bytes(K)
    pk = torch.zeros((max(T, 1), hb + rb), dtype=torch.uint8, device=H.DEV)
    ctx.mw_pack_packets(H.dev(codes), H.dev(scales), tk_d, sb.mask, sb.perm, sb.stats, pk)
    want_pk = ref.pack_packets(codes, scales, tk, mask, perm)
    H.assert_same_bytes(H.host(pk)[:N], want_pk, "packets")
    kids = [torch.zeros((max(T, 1), hb + rb), dtype=torch.uint8, device=H.DEV) for _ in range(n_hops)]
    table = torch.tensor([k.data_ptr() for k in kids], dtype=torch.int64, device=H.DEV)
    stats = torch.zeros(B.RELAY_STATS_BYTES, dtype=torch.uint8, device=H.DEV)
    ctx.mw_relay_packets(B.packets_table([pk], [N], H.DEV), table, max(T, 1), stats)
    pst = ctx.mw_get_relay_stats(stats)
    assert int(pst["error_flags"]) == 0
    for h in range(n_hops):
        want, copies, dests = ref.relay_packets_child(want_pk, next_hop, n_hops, h)
        n = int(pst["rows_per_hop"][h])
        assert n == len(want)
        H.assert_same_bytes(H.host(kids[h])[:n], want, "child %d packets" % h)
    if N:
        assert int(pst["forward_bytes"]) == copies * (hb + rb) and int(pst["unicast_bytes"]) == dests * (hb + rb)
    ctx.close()
