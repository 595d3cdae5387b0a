"""Glue for the GPU parity tests: runs the HIP path through the C-ABI binding on
seeded inputs and hands back host copies, and runs the CPU oracle on the same
inputs.  The two pipelines never exchange intermediate results."""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle import ref
from paper_2605_22428_amd import binding as B
from paper_2605_22428_amd import workloads as W

DEV = "cuda:0"


def fmt_code(w: W.DispatchWorkload) -> int:
    return B.MW_ROW_BF16 if w.row_format == "bf16" else B.MW_ROW_FP8_E4M3_BLOCK128


def make_ctx(w: W.DispatchWorkload, my_rank: Optional[int] = None, max_recv_rows: Optional[int] = None,
             max_tokens: Optional[int] = None, row_stride: int = 0) -> B.Context:
    r = w.my_rank if my_rank is None else my_rank
    cap = max_recv_rows if max_recv_rows is not None else w.n_ranks * w.n_tokens
    return B.Context(w.n_ranks, w.n_experts, w.top_k, r, w.hidden, fmt_code(w),
                     max_tokens if max_tokens is not None else max(w.n_tokens, 1), cap,
                     W.expert_to_rank(w), device=DEV, row_stride=row_stride)


_SIGNED = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32, np.dtype(np.uint64): np.int64}


def dev(a: Optional[np.ndarray]) -> Optional[torch.Tensor]:
    """Upload; unsigned 16/32/64-bit arrays travel as the signed type of the same width."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype in _SIGNED:
        a = a.view(_SIGNED[a.dtype])
    return torch.from_numpy(a).to(DEV)


def host(t: torch.Tensor, dtype=None) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a if dtype is None else a.view(dtype)


class GpuSend:
    """mw_plan + mw_pack (or the single-launch mw_plan_pack) of one rank's tokens; host copies
    of everything written."""

    def __init__(self, ctx: B.Context, topk: np.ndarray, x: np.ndarray, scales: Optional[np.ndarray],
                 x_dev: Optional[torch.Tensor] = None, scales_dev: Optional[torch.Tensor] = None,
                 fused: bool = False, prefill: int = 0):
        self.ctx, self.T, self.prefill = ctx, topk.shape[0], prefill
        self.topk_d = dev(topk.astype(np.int32))
        self.x_d = x_dev if x_dev is not None else dev(x)
        self.s_d = scales_dev if scales_dev is not None else dev(scales)
        self.buf = B.SendBuffers(ctx, self.T)
        if prefill:          # a row the packer misses, or writes to the wrong place, then shows as the pattern
            self.buf.packed.fill_(prefill)
            self.buf.row_src_token.fill_(-prefill)
            self.buf.row_topk.fill_(-prefill)
        if fused:
            ctx.mw_plan_pack(self.topk_d, self.x_d, self.s_d, self.buf.mask, self.buf.perm, self.buf.desc,
                             self.buf.stats, self.buf.packed, self.buf.row_src_token, self.buf.row_topk)
        else:
            ctx.mw_plan(self.topk_d, self.buf.mask, self.buf.perm, self.buf.desc, self.buf.stats)
            ctx.mw_pack(self.x_d, self.s_d, self.topk_d, self.buf.perm, self.buf.stats, self.buf.packed,
                        self.buf.row_src_token, self.buf.row_topk)
        self.stats = ctx.mw_get_send_stats(self.buf.stats)
        self.N, self.G = int(self.stats["n_rows"]), int(self.stats["n_groups"])

    def host_plan(self):
        b = self.buf
        mask = host(b.mask).view(np.uint64)[: self.T]
        perm = host(b.perm)[: self.N]
        desc = host(b.desc).reshape(-1).view(B.DESC_DTYPE)[: self.G]
        return mask, perm, desc

    def host_pack(self):
        b = self.buf
        return (host(b.packed)[: self.N, : self.ctx.row_bytes], host(b.row_src_token)[: self.N],
                host(b.row_topk)[: self.N])

    def deliver(self, dst_rank: int) -> dict:
        """mw_sim_deliver -> record for peers_table (device tensors, counts read back)."""
        ctx, b, n = self.ctx, self.buf, max(self.T, 1)
        out = dict(desc=torch.zeros((n, B.DESC_BYTES), dtype=torch.uint8, device=DEV),
                   rows=torch.zeros((n, ctx.row_stride), dtype=torch.uint8, device=DEV),
                   row_src_token=torch.full((n,), -1, dtype=torch.int32, device=DEV),
                   row_topk=torch.zeros((n, ctx.top_k), dtype=torch.int32, device=DEV))
        counts = torch.zeros(2, dtype=torch.int32, device=DEV)
        ctx.mw_sim_deliver(b.desc, b.stats, self.T, b.packed, b.row_src_token, b.row_topk, dst_rank,
                           out["desc"], out["rows"], out["row_src_token"], out["row_topk"], counts)
        c = counts.cpu().numpy()
        out["n_desc"], out["n_rows"] = int(c[0]), int(c[1])
        return out

    def full_record(self) -> dict:
        b = self.buf
        return dict(desc=b.desc, rows=b.packed, row_src_token=b.row_src_token, row_topk=b.row_topk,
                    n_desc=self.G, n_rows=self.N)


def record_host(rec: dict, row_bytes: Optional[int] = None):
    """Host copy of a peer record as the oracle's (desc, rows, src_token, row_topk) tuple
    (row_bytes: the rows' own length where the record's rows are further apart)."""
    g, n = rec["n_desc"], rec["n_rows"]
    return (host(rec["desc"]).reshape(-1).view(B.DESC_DTYPE)[:g], host(rec["rows"])[:n, :row_bytes],
            host(rec["row_src_token"])[:n], host(rec["row_topk"])[:n])


def shrink(rec: dict) -> dict:
    """Keep only the used prefix of a delivered record (frees the capacity-sized buffers)."""
    g, n = rec["n_desc"], rec["n_rows"]
    return dict(desc=rec["desc"][: max(g, 1)].clone(), rows=rec["rows"][: max(n, 1)].clone(),
                row_src_token=rec["row_src_token"][: max(n, 1)].clone(),
                row_topk=rec["row_topk"][: max(n, 1)].clone(), n_desc=g, n_rows=n)


def oracle_send(w: W.DispatchWorkload, topk: np.ndarray, x: np.ndarray, scales):
    """The oracle's own send side: (desc, packed rows, row_src_token, row_topk).  What the oracle
    is given further down the path (delivery, relay, unpack) is always this, never a GPU buffer."""
    _, perm, desc, _ = ref.plan(topk, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    packed, src, rtk = ref.pack(x, scales, topk, perm)
    return desc, packed, src, rtk


def oracle_packets(w: W.DispatchWorkload, topk: np.ndarray, x: np.ndarray, scales) -> np.ndarray:
    """The oracle's own packets of one sender."""
    mask, perm, _, _ = ref.plan(topk, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    return ref.pack_packets(x, scales, topk, mask, perm)


class GpuUnpack:
    def __init__(self, ctx: B.Context, records: Sequence[dict], capacity: int):
        self.ctx = ctx
        self.table = B.peers_table(records, DEV)
        self.buf = B.RecvBuffers(ctx, capacity)
        b = self.buf
        ctx.mw_unpack(self.table, len(records), b.out_rows, b.out_scales, capacity, b.out_src_peer,
                      b.out_src_token, b.expert_offsets, b.stats)
        self.stats = ctx.mw_get_recv_stats(b.stats)
        self.Q = int(self.stats["n_out_rows"])

    def host_out(self):
        b, q = self.buf, min(self.Q, self.buf.capacity)
        return (host(b.out_rows)[:q], None if b.out_scales is None else host(b.out_scales)[:q],
                host(b.out_src_peer)[:q], host(b.out_src_token)[:q], host(b.expert_offsets))


def assert_same_bytes(a: np.ndarray, b: np.ndarray, what: str):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    assert a.shape == b.shape, "%s: shape %s vs %s" % (what, a.shape, b.shape)
    if a.tobytes() != b.tobytes():
        av, bv = a.reshape(-1).view(np.uint8), b.reshape(-1).view(np.uint8)
        bad = np.nonzero(av != bv)[0]
        raise AssertionError("%s: %d differing bytes, first at %d" % (what, len(bad), int(bad[0])))


def check_send(w: W.DispatchWorkload, g: GpuSend, topk: np.ndarray, x: np.ndarray, scales):
    """Bit-exact comparison of mw_plan / mw_pack output with the oracle."""
    e2r = W.expert_to_rank(w)
    m, perm, desc, st = ref.plan(topk, e2r, w.n_ranks, w.row_bytes)
    gm, gperm, gdesc = g.host_plan()
    assert_same_bytes(gm, m, "mask")
    assert_same_bytes(gperm, perm, "perm")
    assert_same_bytes(gdesc.view(np.uint8), desc.view(np.uint8), "desc")
    assert int(g.stats["error_flags"]) == 0
    for f in ("n_rows", "n_groups", "multicast_bytes", "unicast_bytes"):
        assert int(g.stats[f]) == int(st[f]), f
    assert_same_bytes(g.stats["rows_per_dest"], st["rows_per_dest"], "rows_per_dest")
    packed, src, rtk = ref.pack(x, scales, topk, perm)
    gp, gs, gt = g.host_pack()
    assert_same_bytes(gp, packed, "packed rows")
    if g.ctx.row_stride > g.ctx.row_bytes:                 # the bytes between rows are never written
        assert (host(g.buf.packed)[: g.N, g.ctx.row_bytes:] == g.prefill).all(), "bytes between packed rows were written"
    if g.prefill and g.N < g.T:                            # nor are the rows behind the last packed one
        assert (host(g.buf.packed)[g.N:] == g.prefill).all(), "rows behind the last packed row were written"
    assert_same_bytes(gs, src, "row_src_token")
    assert_same_bytes(gt, rtk, "row_topk")
    return perm, desc, packed, src, rtk


def check_unpack(gu: GpuUnpack, expect, what: str = "unpack"):
    """expect = oracle (out_rows, out_scales, src_peer, src_token, expert_offsets[, M])."""
    o = gu.host_out()
    assert int(gu.stats["error_flags"]) == 0, hex(int(gu.stats["error_flags"]))
    assert_same_bytes(o[4], expect[4], what + " expert_offsets")
    assert_same_bytes(o[2], expect[2], what + " out_src_peer")
    assert_same_bytes(o[3], expect[3], what + " out_src_token")
    assert_same_bytes(o[0], expect[0], what + " out_rows")
    if expect[1] is not None:
        assert_same_bytes(o[1], expect[1], what + " out_scales")
    if len(expect) > 5:
        assert int(gu.stats["n_recv_rows"]) == expect[5]
