"""GPU parity of the steps of SMALL batches (Section 6.3's batch sizes, 64 and 128 tokens a rank):
mw_stream_step, mw_unpack_expand_index_plan_next and mw_unpack_expand_index_next at sizes where
the next batch's index and plan run in one workgroup each.  Every output against the oracle on
the same seeded inputs, bit-exact; and, on inconsistent inputs, the one-workgroup index against
the library's own general index (mw_unpack), flag by flag."""
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


def _check_plan(w, ctx, sb, tk, what):
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


SHAPES = {
    # the decode-sized batches of the dispatch experiment at the paper's row size
    "c1_64": (W.scaled(W.C1, n_tokens=64), 0, None),
    "c1_128": (W.scaled(W.C1, n_tokens=128, hidden=1024), 9, None),
    "fp8_64": (W.scaled(W.C2, n_tokens=64, hidden=1024), 40, None),
    # few peers: at most 480 rows, two rows a lane
    "r8": (W.DispatchWorkload("r8", 61, 8, 16, 2, 60, 256, "bf16", "uniform"), 3, None),
    # every token of every peer comes here: 2000 rows, more than a lane keeps in registers
    "hot": (W.DispatchWorkload("hot", 62, 8, 16, 4, 250, 256, "bf16", "uniform"), 5, "hot"),
    # bitmaps of two and four words (short keys), and more than eight ids a token (no short keys)
    "r128": (W.DispatchWorkload("r128", 63, 128, 256, 8, 40, 256, "bf16", "uniform"), 77, None),
    "r256": (W.scaled(W.C3, n_tokens=24, hidden=256), 200, None),
    "c3_64": (W.scaled(W.C3, n_tokens=64, hidden=256), 17, None),
    "k12": (W.DispatchWorkload("k12", 64, 4, 64, 12, 100, 256, "bf16", "uniform"), 1, None),
    "k9_r130": (W.DispatchWorkload("k9", 65, 130, 260, 9, 30, 256, "bf16", "uniform"), 100, None),
}


@pytest.mark.parametrize("which", sorted(SHAPES))
def test_small_stream_steps_match_the_oracle(which):
    w, my_rank, route = SHAPES[which]
    _say("small steps", which, "R", w.n_ranks, "T", w.n_tokens, "K", w.top_k, "H", w.hidden, w.row_format)
    e2r = W.expert_to_rank(w)
    T, R = w.n_tokens, w.n_ranks
    mine = int(np.nonzero(e2r == my_rank)[0][0])
    ctxs = [H.make_ctx(w, my_rank), H.make_ctx(w, my_rank)]
    n_steps = 3
    batches = []
    for seed in range(1, n_steps + 2):
        recs, toks = [], []
        for p in range(R):
            tk = W.topk_ids(w, seed, p)
            if route == "hot":
                tk[:, 0] = mine
                for j in range(1, w.top_k):                 # (an id is named once per token)
                    tk[tk[:, j] == mine, j] = -1
            if seed == 2 and p == 1:
                tk[:] = -1                                  # a peer that sends nothing
            x, sc = W.payload_rows(w, seed, p)
            recs.append(H.shrink(H.GpuSend(ctxs[0], tk, x, sc).deliver(my_rank)))
            toks.append((tk, x, sc))
        cap = max(1, sum(r["n_rows"] for r in recs) * min(w.top_k, w.experts_per_rank))
        batches.append(dict(recs=recs, toks=toks, cap=cap, table=B.peers_table(recs, H.DEV)))
    sends = []
    for j in range(n_steps + 1):
        tk = W.topk_ids(w, 30 + j, my_rank)
        if j == 2:
            tk[::3] = -1
        x, sc = W.payload_rows(w, 30 + j, my_rank)
        sends.append(dict(tk=tk, x=x, sc=sc, tk_d=H.dev(tk), x_d=H.dev(x), s_d=H.dev(sc), buf=B.SendBuffers(ctxs[0], T)))
    bufs = [B.RecvBuffers(ctxs[i % 2], b["cap"]) for i, b in enumerate(batches)]
    s0 = sends[0]
    ctxs[0].mw_plan(s0["tk_d"], s0["buf"].mask, s0["buf"].perm, s0["buf"].desc, s0["buf"].stats)
    ctxs[0].mw_unpack_index(batches[0]["table"], R, batches[0]["cap"], bufs[0].expert_offsets, bufs[0].stats)
    for i in range(n_steps):
        cur, nxt = ctxs[i % 2], ctxs[(i + 1) % 2]
        sd, sn = sends[i], sends[i + 1]
        b, nb = batches[i], batches[i + 1]
        if i == 1:      # the two-launch form of the same step
            cur.mw_pack(sd["x_d"], sd["s_d"], sd["tk_d"], sd["buf"].perm, sd["buf"].stats, sd["buf"].packed,
                        sd["buf"].row_src_token, sd["buf"].row_topk)
            cur.mw_unpack_expand_index_plan_next(R, bufs[i].out_rows, bufs[i].out_scales, b["cap"], bufs[i].out_src_peer,
                                                 bufs[i].out_src_token, nxt, nb["table"], R, nb["cap"],
                                                 bufs[i + 1].expert_offsets, bufs[i + 1].stats, sn["tk_d"],
                                                 sn["buf"].mask, sn["buf"].perm, sn["buf"].desc, sn["buf"].stats)
        else:
            cur.mw_stream_step(sd["x_d"], sd["s_d"], sd["tk_d"], sd["buf"].perm, sd["buf"].stats, sd["buf"].packed,
                               sd["buf"].row_src_token, sd["buf"].row_topk, R, bufs[i].out_rows, bufs[i].out_scales,
                               b["cap"], bufs[i].out_src_peer, bufs[i].out_src_token, nxt, nb["table"], R, nb["cap"],
                               bufs[i + 1].expert_offsets, bufs[i + 1].stats, sn["tk_d"], sn["buf"].mask, sn["buf"].perm,
                               sn["buf"].desc, sn["buf"].stats)
        if i == 0:      # from here on the contexts know how many rows to expect
            torch.cuda.synchronize()
            nxt.mw_get_recv_stats(bufs[i + 1].stats)
    torch.cuda.synchronize()
    for i in range(n_steps):
        b = batches[i]
        want = ref.dispatch_plain(b["toks"], e2r, my_rank, b["cap"])
        st = ctxs[i % 2].mw_get_recv_stats(bufs[i].stats)
        q = int(st["n_out_rows"])
        assert int(st["error_flags"]) == 0 and q == len(want[2])
        assert int(st["n_recv_rows"]) == sum(len(W.tokens_for_rank(w, t[0], my_rank)) for t in b["toks"])
        assert int(st["n_rows_seen"]) == sum(r["n_rows"] for r in b["recs"])
        H.assert_same_bytes(H.host(bufs[i].expert_offsets), want[4], "step %d expert_offsets" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_peer)[:q], want[2], "step %d out_src_peer" % i)
        H.assert_same_bytes(H.host(bufs[i].out_src_token)[:q], want[3], "step %d out_src_token" % i)
        H.assert_same_bytes(H.host(bufs[i].out_rows)[:q], want[0], "step %d out_rows" % i)
        if want[1] is not None:
            H.assert_same_bytes(H.host(bufs[i].out_scales)[:q], want[1], "step %d out_scales" % i)
    for j in range(n_steps + 1):
        sd = sends[j]
        _check_plan(w, ctxs[0], sd["buf"], sd["tk"], "send batch %d" % j)
        if j < n_steps:
            _, perm, _, _ = ref.plan(sd["tk"], e2r, R, w.row_bytes)
            packed, src, rtk = ref.pack(sd["x"], sd["sc"], sd["tk"], perm)
            n = len(perm)
            H.assert_same_bytes(H.host(sd["buf"].packed)[:n], packed, "send batch %d packed rows" % j)
            H.assert_same_bytes(H.host(sd["buf"].row_src_token)[:n], src, "send batch %d row_src_token" % j)
            H.assert_same_bytes(H.host(sd["buf"].row_topk)[:n], rtk, "send batch %d row_topk" % j)
    for c in ctxs:
        c.close()


# ---------------------------------------------------------------- inconsistent inputs
W_ERR = W.DispatchWorkload("small_err", 71, 8, 16, 2, 96, 256, "bf16", "uniform")
ERR_RANK = 3


def _regions(ctx, seed=4):
    recs = []
    for p in range(W_ERR.n_ranks):
        tk = W.topk_ids(W_ERR, seed, p)
        x, _ = W.payload_rows(W_ERR, seed, p)
        recs.append(H.shrink(H.GpuSend(ctx, tk, x, None).deliver(ERR_RANK)))
    return recs


def _damage(recs, case):
    e2r = W.expert_to_rank(W_ERR)
    if case == "bad_src_token":
        recs[1]["row_src_token"][0] = W_ERR.n_tokens + 5
        recs[4]["row_src_token"][2] = -3
    elif case == "no_local_expert":
        elsewhere = int(np.nonzero(e2r != ERR_RANK)[0][0])
        recs[2]["row_topk"][1] = torch.tensor([elsewhere, -1], dtype=torch.int32)
    elif case == "bad_expert":
        row_tk = H.host(recs[5]["row_topk"])[0]
        keep = [int(e) for e in row_tk if e >= 0 and e2r[e] == ERR_RANK]
        recs[5]["row_topk"][0] = torch.tensor([keep[0], W_ERR.n_experts + 7], dtype=torch.int32)
    elif case == "bad_desc":
        d = H.host(recs[6]["desc"]).reshape(-1).view(B.DESC_DTYPE).copy()
        d["row_count"][recs[6]["n_desc"] - 1] += 1000
        recs[6]["desc"] = H.dev(d.view(np.uint8).reshape(-1, B.DESC_BYTES))
    elif case == "dup_src_token":
        src = H.host(recs[0]["row_src_token"])
        rtk = H.host(recs[0]["row_topk"])
        local = lambda row: {int(e) for e in rtk[row] if e >= 0 and e2r[e] == ERR_RANK}
        a, b = next((a, b) for a in range(len(src)) for b in range(a + 1, len(src)) if local(a) & local(b))
        recs[0]["row_src_token"][b] = int(src[a])
    return recs


@pytest.mark.parametrize("case", ["clean", "bad_src_token", "no_local_expert", "bad_expert", "bad_desc", "dup_src_token",
                                  "recv_capacity", "max_tokens", "out_capacity"])
def test_one_workgroup_index_reports_what_the_general_index_reports(case):
    """The same (damaged) regions through mw_unpack -- one workgroup per peer, counts exchanged --
    and through the index that rides in a small step's launch: statistics, flags, expert offsets
    and everything delivered must be the same (what is delivered for a repeated source token is
    unspecified: flags and statistics only there)."""
    w = W_ERR
    kw = {}
    full = _regions(H.make_ctx(w, ERR_RANK))
    total = sum(r["n_rows"] for r in full)
    if case == "recv_capacity":
        kw["max_recv_rows"] = total // 2
    if case == "max_tokens":
        kw["max_tokens"] = 8
    gen = H.make_ctx(w, ERR_RANK, **kw)
    a, b = H.make_ctx(w, ERR_RANK, **kw), H.make_ctx(w, ERR_RANK, **kw)
    recs = _damage(_regions(H.make_ctx(w, ERR_RANK)), case)
    cap = 4 * total if case != "out_capacity" else max(1, total // 3)
    gu = H.GpuUnpack(gen, recs, cap)
    # something for context a to expand: the clean regions
    clean = _regions(H.make_ctx(w, ERR_RANK))
    ta, tb = B.peers_table(clean, H.DEV), B.peers_table(recs, H.DEV)
    ra, rb = B.RecvBuffers(a, 4 * total), B.RecvBuffers(b, cap)
    R = w.n_ranks
    a.mw_unpack_index(ta, R, 4 * total, ra.expert_offsets, ra.stats)
    a.mw_unpack_expand_index_next(R, ra.out_rows, ra.out_scales, 4 * total, ra.out_src_peer, ra.out_src_token, b, tb, R,
                                  cap, rb.expert_offsets, rb.stats)
    b.mw_unpack_expand(R, rb.out_rows, rb.out_scales, cap, rb.out_src_peer, rb.out_src_token)
    st = b.mw_get_recv_stats(rb.stats)
    for f in ("n_recv_rows", "n_out_rows", "error_flags", "n_rows_seen"):
        assert int(st[f]) == int(gu.stats[f]), (case, f, int(st[f]), int(gu.stats[f]))
    want_flag = {"clean": 0, "bad_src_token": B.MW_FLAG_BAD_SRC_TOKEN, "no_local_expert": B.MW_FLAG_NO_LOCAL_EXPERT,
                 "bad_expert": B.MW_FLAG_BAD_EXPERT, "bad_desc": B.MW_FLAG_BAD_DESC,
                 "dup_src_token": B.MW_FLAG_DUP_SRC_TOKEN, "out_capacity": B.MW_FLAG_OUT_CAPACITY}.get(case)
    if want_flag is not None:
        assert int(st["error_flags"]) == want_flag, hex(int(st["error_flags"]))
    else:
        assert int(st["error_flags"]) & B.MW_FLAG_RECV_CAPACITY
    H.assert_same_bytes(H.host(rb.expert_offsets), H.host(gu.buf.expert_offsets), "expert_offsets")
    if case != "dup_src_token":
        q = min(int(st["n_out_rows"]), cap)
        H.assert_same_bytes(H.host(rb.out_src_peer)[:q], H.host(gu.buf.out_src_peer)[:q], "out_src_peer")
        H.assert_same_bytes(H.host(rb.out_src_token)[:q], H.host(gu.buf.out_src_token)[:q], "out_src_token")
        H.assert_same_bytes(H.host(rb.out_rows)[:q], H.host(gu.buf.out_rows)[:q], "out_rows")
    # the flags do not stick: a clean batch through the same contexts reports none
    b.mw_unpack_index(ta, R, 4 * total, ra.expert_offsets, ra.stats)
    b.mw_unpack_expand_index_next(R, ra.out_rows, ra.out_scales, 4 * total, ra.out_src_peer, ra.out_src_token, a, ta, R,
                                  4 * total, ra.expert_offsets, ra.stats)
    st2 = a.mw_get_recv_stats(ra.stats)
    if case not in ("recv_capacity", "max_tokens"):
        assert int(st2["error_flags"]) == 0
    for c in (gen, a, b):
        c.close()
