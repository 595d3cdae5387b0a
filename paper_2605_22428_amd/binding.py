"""Thin Python binding of libmw.so (the C ABI declared in include/mw.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
the shared library.  PyTorch is used for device memory and streams, nothing
else.  There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmw.so")

MW_OK = 0
MW_ERR_INVALID_ARG, MW_ERR_CAPACITY, MW_ERR_UNSUPPORTED, MW_ERR_HIP, MW_ERR_WORKSPACE = -1, -2, -3, -4, -5
MW_ROW_BF16, MW_ROW_FP8_E4M3_BLOCK128, MW_ROW_BYTES = 0, 1, 2
MW_FLAG_BAD_EXPERT, MW_FLAG_OUT_CAPACITY, MW_FLAG_NO_LOCAL_EXPERT = 0x01, 0x02, 0x04
MW_FLAG_BAD_SRC_TOKEN, MW_FLAG_BAD_DESC, MW_FLAG_RECV_CAPACITY, MW_FLAG_DUP_SRC_TOKEN = 0x08, 0x10, 0x20, 0x40

EXPORTS = ["mw_workspace_bytes", "mw_ctx_create", "mw_ctx_destroy", "mw_plan", "mw_pack", "mw_plan_pack", "mw_pack_quantize",
           "mw_packet_header_bytes", "mw_pack_packets", "mw_unpack_packets",
           "mw_plan_allgather", "mw_pack_allgather", "mw_unpack", "mw_unpack_index", "mw_unpack_expand",
           "mw_unpack_allgather", "mw_combine_gather", "mw_unpack_expand_index_next", "mw_unpack_expand_index_plan_next", "mw_ctx_set_ride_wait_limit", "mw_stream_step", "mw_allgather_step",
           "mw_sim_deliver", "mw_copy_bytes", "mw_get_send_stats", "mw_get_recv_stats",
           "mw_set_forwarding", "mw_relay", "mw_relay_index", "mw_relay_copy", "mw_relay_copy_index_next", "mw_relay_packets", "mw_relay_packets_index", "mw_relay_packets_copy", "mw_relay_packets_copy_index_next", "mw_get_relay_stats",
           "mw_allgather_split_point", "mw_plan_allgather_split", "mw_unpack_allgather_split",
           "mw_ctx_set_timing_events", "mw_status_string", "mw_plan_static", "mw_ctx_set_options", "mw_relay_batch"]
MW_KERNEL_PLAN_RANK, MW_KERNEL_PLAN_GROUPS, MW_KERNEL_PACK, MW_KERNEL_RECV_INDEX, MW_KERNEL_EXPAND = 0, 1, 2, 3, 4
MW_KERNEL_AG_PACK, MW_KERNEL_AG_GATHER, MW_KERNEL_RELAY_INDEX, MW_KERNEL_RELAY_COPY = 5, 6, 7, 8
MW_KERNEL_PLAN_PACK, MW_KERNEL_PACK_QUANT, MW_KERNEL_COMBINE = 9, 10, 11
MW_MAX_HOPS = 64
MW_FUSED_MAX_TOKENS = 256
MW_RIDE_MAX_TOKENS = 8192
MW_STATIC_MAX_TOKENS, MW_STATIC_MAX_EXPERTS = 8192, 1024
MW_FLAG_BAD_RANK = 0x80
MW_FLAG_PLAN_TIMEOUT = 0x100
MW_FLAG_DUPLICATE_DROPPED = 0x200
MW_OPT_RELAY_KEEP_METADATA, MW_OPT_RECV_DEDUP = 0x1, 0x2

# numpy views of the ABI records (host copies)
DESC_DTYPE = np.dtype([("mask", "<u8", (4,)), ("row_offset", "<u4"), ("row_count", "<u4"),
                       ("n_dest", "<u4"), ("reserved0", "<u4")])
SEND_STATS_DTYPE = np.dtype([("n_rows", "<u4"), ("n_groups", "<u4"), ("multicast_bytes", "<u8"),
                             ("unicast_bytes", "<u8"), ("rows_per_dest", "<u4", (256,)),
                             ("error_flags", "<u4"), ("reserved0", "<u4")])
RECV_STATS_DTYPE = np.dtype([("n_recv_rows", "<u8"), ("n_out_rows", "<u8"), ("error_flags", "<u4"),
                             ("n_rows_seen", "<u4")])
RECV_PEER_DTYPE = np.dtype([("desc", "<u8"), ("n_desc", "<u4"), ("n_rows", "<u4"), ("rows", "<u8"),
                            ("row_src_token", "<u8"), ("row_topk", "<u8")])
RECV_PACKETS_DTYPE = np.dtype([("packets", "<u8"), ("n_rows", "<u4"), ("reserved0", "<u4")])
RELAY_CHILD_DTYPE = np.dtype([("desc", "<u8"), ("rows", "<u8"), ("row_src_token", "<u8"), ("row_topk", "<u8")])
RELAY_STATS_DTYPE = np.dtype([("n_groups_in", "<u4"), ("n_rows_in", "<u4"), ("forward_bytes", "<u8"),
                              ("unicast_bytes", "<u8"), ("groups_per_hop", "<u4", (64,)),
                              ("rows_per_hop", "<u4", (64,)), ("error_flags", "<u4"), ("reserved0", "<u4")])
DESC_BYTES, SEND_STATS_BYTES, RECV_STATS_BYTES, RECV_PEER_BYTES = 48, 1056, 24, 40
RELAY_CHILD_BYTES, RELAY_STATS_BYTES = 32, 544
assert (RELAY_CHILD_DTYPE.itemsize, RELAY_STATS_DTYPE.itemsize) == (32, 544)
assert (DESC_DTYPE.itemsize, SEND_STATS_DTYPE.itemsize, RECV_STATS_DTYPE.itemsize,
        RECV_PEER_DTYPE.itemsize) == (48, 1056, 24, 40)


class MwConfig(C.Structure):
    _fields_ = [("n_ranks", C.c_int32), ("n_experts", C.c_int32), ("top_k", C.c_int32),
                ("my_rank", C.c_int32), ("hidden", C.c_int32), ("row_format", C.c_int32),
                ("row_bytes", C.c_int64), ("max_tokens", C.c_int32), ("max_hops", C.c_int32),
                ("max_recv_rows", C.c_int64), ("expert_to_rank", C.c_void_p), ("row_stride_bytes", C.c_int64)]


class MwSendBatch(C.Structure):
    """mw_send_batch (include/mw.h)."""
    _fields_ = [("x_dev", C.c_void_p), ("scales_dev", C.c_void_p), ("topk_ids_dev", C.c_void_p),
                ("perm_dev", C.c_void_p), ("stats_dev", C.c_void_p), ("packed_rows_dev", C.c_void_p),
                ("row_src_token_dev", C.c_void_p), ("row_topk_dev", C.c_void_p), ("n_tokens", C.c_int32),
                ("reserved0", C.c_int32)]


class MwRecvBatch(C.Structure):
    """mw_recv_batch (include/mw.h)."""
    _fields_ = [("out_rows_dev", C.c_void_p), ("out_scales_dev", C.c_void_p), ("out_src_peer_dev", C.c_void_p),
                ("out_src_token_dev", C.c_void_p), ("out_capacity_rows", C.c_int64), ("n_peers", C.c_int32),
                ("reserved0", C.c_int32)]


class MwNextBatch(C.Structure):
    """mw_next_batch (include/mw.h)."""
    _fields_ = [("ctx", C.c_void_p), ("peers_dev", C.c_void_p), ("expert_offsets_dev", C.c_void_p),
                ("recv_stats_dev", C.c_void_p), ("out_capacity_rows", C.c_int64), ("n_peers", C.c_int32),
                ("n_tokens", C.c_int32), ("topk_ids_dev", C.c_void_p), ("mask_dev", C.c_void_p),
                ("perm_dev", C.c_void_p), ("desc_dev", C.c_void_p), ("send_stats_dev", C.c_void_p)]


class MwRelayJob(C.Structure):
    """mw_relay_job (include/mw.h)."""
    _fields_ = [("ctx", C.c_void_p), ("in_dev", C.c_void_p), ("children_dev", C.c_void_p),
                ("child_capacity_rows", C.c_int64), ("stats_dev", C.c_void_p)]


class MwError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))
        self.status = status


_lib = None


def load():
    """Load libmw.so (built by paper_2605_22428_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is not built (run __graft_entry__.build())" % LIB_PATH)
        lib = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = C.c_int32
        lib.mw_status_string.restype = C.c_char_p
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().mw_status_string(C.c_int32(status)).decode()


def _check(status: int, where: str):
    if status != MW_OK:
        raise MwError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def mw_copy_bytes(dst: torch.Tensor, src: torch.Tensor, n_bytes: int):
    _check(load().mw_copy_bytes(_ptr(dst), _ptr(src), C.c_int64(n_bytes), _stream()), "mw_copy_bytes")


def mw_packet_header_bytes(top_k: int) -> int:
    a = C.c_int64(0)
    _check(load().mw_packet_header_bytes(C.c_int32(top_k), C.byref(a)), "mw_packet_header_bytes")
    return a.value


def mw_allgather_split_point(shard_bytes: int, bw_direct: float, bw_relay: float, copies: int) -> int:
    a = C.c_int64(0)
    _check(load().mw_allgather_split_point(C.c_int64(shard_bytes), C.c_double(bw_direct), C.c_double(bw_relay),
                                           C.c_int32(copies), C.byref(a)), "mw_allgather_split_point")
    return a.value


def mw_plan_static(n_ranks: int, n_experts: int, top_k: int, hidden: int, row_format: int, row_bytes: int,
                   expert_to_rank: torch.Tensor, topk_ids: torch.Tensor, mask: torch.Tensor, perm: torch.Tensor,
                   desc: torch.Tensor, stats: torch.Tensor):
    """mw_plan without a context or a workspace; expert_to_rank is a device tensor of int32."""
    cfg = MwConfig(n_ranks, n_experts, top_k, 0, hidden, row_format, row_bytes, 0, 0, 0, 0, 0)
    _check(load().mw_plan_static(C.byref(cfg), _ptr(expert_to_rank), _ptr(topk_ids), C.c_int32(topk_ids.shape[0]),
                                 _ptr(mask), _ptr(perm), _ptr(desc), _ptr(stats), _stream()), "mw_plan_static")


def _addr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.data_ptr()


def send_batch(x, scales, topk_ids, perm, stats, packed, row_src_token, row_topk) -> MwSendBatch:
    return MwSendBatch(_addr(x), _addr(scales), _addr(topk_ids), _addr(perm), _addr(stats), _addr(packed),
                       _addr(row_src_token), _addr(row_topk), int(topk_ids.shape[0]), 0)


def recv_batch(n_peers, out_rows, out_scales, out_capacity_rows, out_src_peer, out_src_token) -> MwRecvBatch:
    return MwRecvBatch(_addr(out_rows), _addr(out_scales), _addr(out_src_peer), _addr(out_src_token),
                       int(out_capacity_rows), int(n_peers), 0)


def next_batch(next_ctx, peers, n_peers, out_capacity_rows, expert_offsets, recv_stats, topk_ids=None, mask=None,
               perm=None, desc=None, send_stats=None) -> MwNextBatch:
    return MwNextBatch(next_ctx._h.value if next_ctx is not None else 0, _addr(peers), _addr(expert_offsets),
                       _addr(recv_stats), int(out_capacity_rows), int(n_peers),
                       0 if topk_ids is None else int(topk_ids.shape[0]), _addr(topk_ids), _addr(mask), _addr(perm),
                       _addr(desc), _addr(send_stats))


MW_RELAY_BATCH_MAX = 4


def relay_job(ctx: "Context", in_record: torch.Tensor, children: torch.Tensor, child_capacity_rows: int,
              stats: torch.Tensor) -> MwRelayJob:
    return MwRelayJob(ctx._h.value, _addr(in_record), _addr(children), int(child_capacity_rows), _addr(stats))


def mw_relay_batch(copy_jobs: Sequence[MwRelayJob], index_jobs: Sequence[MwRelayJob]):
    ca = (MwRelayJob * max(len(copy_jobs), 1))(*copy_jobs)
    ia = (MwRelayJob * max(len(index_jobs), 1))(*index_jobs)
    _check(load().mw_relay_batch(ca, C.c_int32(len(copy_jobs)), ia, C.c_int32(len(index_jobs)), _stream()),
           "mw_relay_batch")


class Context:
    """mw_ctx plus the device workspace it uses (a torch tensor, caller-owned in ABI terms)."""

    def __init__(self, n_ranks: int, n_experts: int, top_k: int, my_rank: int, hidden: int,
                 row_format: int, max_tokens: int, max_recv_rows: int,
                 expert_to_rank: Optional[np.ndarray], row_bytes: int = 0, device: str = "cuda:0",
                 max_hops: int = 0, row_stride: int = 0):
        lib = load()
        self.device = torch.device(device)
        e2r = None if expert_to_rank is None else np.ascontiguousarray(expert_to_rank, dtype=np.int32)
        self._e2r = e2r
        cfg = MwConfig(n_ranks, n_experts, top_k, my_rank, hidden, row_format, row_bytes, max_tokens, max_hops,
                       max_recv_rows, 0 if e2r is None else e2r.ctypes.data, row_stride)
        need = C.c_int64(0)
        _check(lib.mw_workspace_bytes(C.byref(cfg), C.byref(need)), "mw_workspace_bytes")
        self.workspace = torch.zeros(need.value + 256, dtype=torch.uint8, device=self.device)
        off = (-self.workspace.data_ptr()) % 256
        handle = C.c_void_p(0)
        with torch.cuda.device(self.device):
            _check(lib.mw_ctx_create(C.byref(cfg), C.c_void_p(self.workspace.data_ptr() + off),
                                     C.c_int64(need.value), C.byref(handle)), "mw_ctx_create")
        self._h = handle
        self.n_ranks, self.n_experts, self.top_k, self.my_rank = n_ranks, n_experts, top_k, my_rank
        self.hidden, self.row_format, self.max_tokens, self.max_recv_rows = hidden, row_format, max_tokens, max_recv_rows
        if row_format == MW_ROW_BF16:
            self.x_row_bytes, self.s_row_bytes = 2 * hidden, 0
        elif row_format == MW_ROW_FP8_E4M3_BLOCK128:
            self.x_row_bytes, self.s_row_bytes = hidden, 4 * (hidden // 128)
        else:
            self.x_row_bytes, self.s_row_bytes = row_bytes, 0
        self.row_bytes = self.x_row_bytes + self.s_row_bytes
        self.row_stride = row_stride if row_stride else self.row_bytes      # bytes from row to row in packed / received arrays
        self.n_local = 0 if e2r is None else int((e2r == my_rank).sum())

    def close(self):
        if self._h is not None and self._h.value:
            load().mw_ctx_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- send side -----------------------------------------------------------------------
    def mw_plan(self, topk_ids: torch.Tensor, mask: torch.Tensor, perm: torch.Tensor,
                desc: torch.Tensor, stats: torch.Tensor):
        n_tokens = topk_ids.shape[0]
        _check(load().mw_plan(self._h, _ptr(topk_ids), C.c_int32(n_tokens), _ptr(mask), _ptr(perm),
                              _ptr(desc), _ptr(stats), _stream()), "mw_plan")

    def mw_pack(self, x: torch.Tensor, scales: Optional[torch.Tensor], topk_ids: torch.Tensor,
                perm: torch.Tensor, stats: torch.Tensor, packed: torch.Tensor,
                row_src_token: torch.Tensor, row_topk: torch.Tensor):
        n_tokens = topk_ids.shape[0]
        _check(load().mw_pack(self._h, _ptr(x), _ptr(scales), _ptr(topk_ids), _ptr(perm), _ptr(stats),
                              C.c_int32(n_tokens), _ptr(packed), _ptr(row_src_token), _ptr(row_topk),
                              _stream()), "mw_pack")

    def mw_pack_quantize(self, x_bf16: torch.Tensor, topk_ids: torch.Tensor, perm: torch.Tensor,
                         stats: torch.Tensor, packed: torch.Tensor, row_src_token: torch.Tensor,
                         row_topk: torch.Tensor):
        n_tokens = topk_ids.shape[0]
        _check(load().mw_pack_quantize(self._h, _ptr(x_bf16), _ptr(topk_ids), _ptr(perm), _ptr(stats),
                                       C.c_int32(n_tokens), _ptr(packed), _ptr(row_src_token), _ptr(row_topk),
                                       _stream()), "mw_pack_quantize")

    def mw_plan_pack(self, topk_ids: torch.Tensor, x: torch.Tensor, scales: Optional[torch.Tensor],
                     mask: torch.Tensor, perm: torch.Tensor, desc: torch.Tensor, stats: torch.Tensor,
                     packed: torch.Tensor, row_src_token: torch.Tensor, row_topk: torch.Tensor):
        n_tokens = topk_ids.shape[0]
        _check(load().mw_plan_pack(self._h, _ptr(topk_ids), _ptr(x), _ptr(scales), C.c_int32(n_tokens), _ptr(mask),
                                   _ptr(perm), _ptr(desc), _ptr(stats), _ptr(packed), _ptr(row_src_token),
                                   _ptr(row_topk), _stream()), "mw_plan_pack")

    def mw_pack_packets(self, x: torch.Tensor, scales: Optional[torch.Tensor], topk_ids: torch.Tensor,
                        mask: torch.Tensor, perm: torch.Tensor, stats: torch.Tensor, packets: torch.Tensor):
        n_tokens = topk_ids.shape[0]
        _check(load().mw_pack_packets(self._h, _ptr(x), _ptr(scales), _ptr(topk_ids), _ptr(mask), _ptr(perm),
                                      _ptr(stats), C.c_int32(n_tokens), _ptr(packets), _stream()), "mw_pack_packets")

    def mw_unpack_packets(self, peers: torch.Tensor, n_peers: int, out_rows: torch.Tensor,
                          out_scales: Optional[torch.Tensor], out_capacity_rows: int, out_src_peer: torch.Tensor,
                          out_src_token: torch.Tensor, expert_offsets: torch.Tensor, recv_stats: torch.Tensor):
        _check(load().mw_unpack_packets(self._h, _ptr(peers), C.c_int32(n_peers), _ptr(out_rows), _ptr(out_scales),
                                        C.c_int64(out_capacity_rows), _ptr(out_src_peer), _ptr(out_src_token),
                                        _ptr(expert_offsets), _ptr(recv_stats), _stream()), "mw_unpack_packets")

    def mw_plan_allgather(self, shard_bytes: int, desc: torch.Tensor, stats: torch.Tensor):
        _check(load().mw_plan_allgather(self._h, C.c_int64(shard_bytes), _ptr(desc), _ptr(stats),
                                        _stream()), "mw_plan_allgather")

    def mw_pack_allgather(self, shard: torch.Tensor, shard_bytes: int, send_buf: torch.Tensor):
        _check(load().mw_pack_allgather(self._h, _ptr(shard), C.c_int64(shard_bytes), _ptr(send_buf),
                                        _stream()), "mw_pack_allgather")

    def mw_plan_allgather_split(self, shard_bytes: int, direct_bytes: int, desc: torch.Tensor, stats: torch.Tensor):
        _check(load().mw_plan_allgather_split(self._h, C.c_int64(shard_bytes), C.c_int64(direct_bytes), _ptr(desc),
                                              _ptr(stats), _stream()), "mw_plan_allgather_split")

    def mw_unpack_allgather_split(self, direct: torch.Tensor, relayed: torch.Tensor, shard_bytes: int,
                                  direct_bytes: int, out: torch.Tensor):
        _check(load().mw_unpack_allgather_split(self._h, _ptr(direct), _ptr(relayed), C.c_int64(shard_bytes),
                                                C.c_int64(direct_bytes), _ptr(out), _stream()),
               "mw_unpack_allgather_split")

    # ---- receive side --------------------------------------------------------------------
    def mw_unpack(self, peers: torch.Tensor, n_peers: int, out_rows: torch.Tensor,
                  out_scales: Optional[torch.Tensor], out_capacity_rows: int, out_src_peer: torch.Tensor,
                  out_src_token: torch.Tensor, expert_offsets: torch.Tensor, recv_stats: torch.Tensor):
        _check(load().mw_unpack(self._h, _ptr(peers), C.c_int32(n_peers), _ptr(out_rows), _ptr(out_scales),
                                C.c_int64(out_capacity_rows), _ptr(out_src_peer), _ptr(out_src_token),
                                _ptr(expert_offsets), _ptr(recv_stats), _stream()), "mw_unpack")

    def mw_unpack_index(self, peers: torch.Tensor, n_peers: int, out_capacity_rows: int,
                        expert_offsets: torch.Tensor, recv_stats: torch.Tensor):
        _check(load().mw_unpack_index(self._h, _ptr(peers), C.c_int32(n_peers), C.c_int64(out_capacity_rows),
                                      _ptr(expert_offsets), _ptr(recv_stats), _stream()), "mw_unpack_index")

    def mw_unpack_expand(self, n_peers: int, out_rows: torch.Tensor, out_scales: Optional[torch.Tensor],
                         out_capacity_rows: int, out_src_peer: torch.Tensor, out_src_token: torch.Tensor):
        _check(load().mw_unpack_expand(self._h, C.c_int32(n_peers), _ptr(out_rows), _ptr(out_scales),
                                       C.c_int64(out_capacity_rows), _ptr(out_src_peer), _ptr(out_src_token),
                                       _stream()), "mw_unpack_expand")

    def mw_unpack_expand_index_next(self, n_peers: int, out_rows: torch.Tensor, out_scales: Optional[torch.Tensor],
                                    out_capacity_rows: int, out_src_peer: torch.Tensor, out_src_token: torch.Tensor,
                                    next_ctx: "Context", next_peers: torch.Tensor, next_n_peers: int,
                                    next_out_capacity_rows: int, next_expert_offsets: torch.Tensor,
                                    next_recv_stats: torch.Tensor):
        recv = recv_batch(n_peers, out_rows, out_scales, out_capacity_rows, out_src_peer, out_src_token)
        nxt = next_batch(next_ctx, next_peers, next_n_peers, next_out_capacity_rows, next_expert_offsets,
                         next_recv_stats)
        _check(load().mw_unpack_expand_index_next(self._h, C.byref(recv), C.byref(nxt), _stream()),
               "mw_unpack_expand_index_next")

    def mw_unpack_expand_index_plan_next(self, n_peers: int, out_rows: torch.Tensor,
                                         out_scales: Optional[torch.Tensor], out_capacity_rows: int,
                                         out_src_peer: torch.Tensor, out_src_token: torch.Tensor,
                                         next_ctx: "Context", next_peers: torch.Tensor, next_n_peers: int,
                                         next_out_capacity_rows: int, next_expert_offsets: torch.Tensor,
                                         next_recv_stats: torch.Tensor, next_topk_ids: torch.Tensor,
                                         next_mask: torch.Tensor, next_perm: torch.Tensor, next_desc: torch.Tensor,
                                         next_send_stats: torch.Tensor):
        recv = recv_batch(n_peers, out_rows, out_scales, out_capacity_rows, out_src_peer, out_src_token)
        nxt = next_batch(next_ctx, next_peers, next_n_peers, next_out_capacity_rows, next_expert_offsets,
                         next_recv_stats, next_topk_ids, next_mask, next_perm, next_desc, next_send_stats)
        _check(load().mw_unpack_expand_index_plan_next(self._h, C.byref(recv), C.byref(nxt), _stream()),
               "mw_unpack_expand_index_plan_next")

    def mw_stream_step(self, x: torch.Tensor, scales: Optional[torch.Tensor], topk_ids: torch.Tensor,
                       perm: torch.Tensor, stats: torch.Tensor, packed: torch.Tensor, row_src_token: torch.Tensor,
                       row_topk: torch.Tensor, n_peers: int, out_rows: torch.Tensor,
                       out_scales: Optional[torch.Tensor], out_capacity_rows: int, out_src_peer: torch.Tensor,
                       out_src_token: torch.Tensor, next_ctx: "Context", next_peers: torch.Tensor,
                       next_n_peers: int, next_out_capacity_rows: int, next_expert_offsets: torch.Tensor,
                       next_recv_stats: torch.Tensor, next_topk_ids: torch.Tensor, next_mask: torch.Tensor,
                       next_perm: torch.Tensor, next_desc: torch.Tensor, next_send_stats: torch.Tensor):
        send = send_batch(x, scales, topk_ids, perm, stats, packed, row_src_token, row_topk)
        recv = recv_batch(n_peers, out_rows, out_scales, out_capacity_rows, out_src_peer, out_src_token)
        nxt = next_batch(next_ctx, next_peers, next_n_peers, next_out_capacity_rows, next_expert_offsets,
                         next_recv_stats, next_topk_ids, next_mask, next_perm, next_desc, next_send_stats)
        _check(load().mw_stream_step(self._h, C.byref(send), C.byref(recv), C.byref(nxt), _stream()),
               "mw_stream_step")

    def mw_stream_step_records(self, send: MwSendBatch, recv: MwRecvBatch, nxt: MwNextBatch,
                               stream_handle: Optional[int] = None):
        """mw_stream_step on records the caller built once (send_batch, recv_batch, next_batch) and keeps,
        together with the tensors they point to: a loop over the same buffers then marshals nothing.
        stream_handle: a stream's raw handle (torch.cuda.Stream.cuda_stream); default: the current stream."""
        st = _stream() if stream_handle is None else C.c_void_p(stream_handle)
        _check(load().mw_stream_step(self._h, C.byref(send), C.byref(recv), C.byref(nxt), st), "mw_stream_step")

    def mw_ctx_set_options(self, options: int):
        _check(load().mw_ctx_set_options(self._h, C.c_uint32(options)), "mw_ctx_set_options")

    def mw_ctx_set_ride_wait_limit(self, polls: int):
        _check(load().mw_ctx_set_ride_wait_limit(self._h, C.c_int64(polls)), "mw_ctx_set_ride_wait_limit")

    def mw_combine_gather(self, n_peers: int, y: torch.Tensor, out_capacity_rows: int, ret_rows: torch.Tensor,
                          ret_capacity_rows: int):
        _check(load().mw_combine_gather(self._h, C.c_int32(n_peers), _ptr(y), C.c_int64(out_capacity_rows),
                                        _ptr(ret_rows), C.c_int64(ret_capacity_rows), _stream()), "mw_combine_gather")

    def mw_unpack_allgather(self, peer_shards: torch.Tensor, shard_bytes: int, out: torch.Tensor):
        _check(load().mw_unpack_allgather(self._h, _ptr(peer_shards), C.c_int64(shard_bytes), _ptr(out),
                                          _stream()), "mw_unpack_allgather")

    def mw_allgather_step(self, shard: torch.Tensor, shard_bytes: int, send_buf: torch.Tensor, desc: torch.Tensor,
                          stats: torch.Tensor, peer_shards: torch.Tensor, out: torch.Tensor):
        _check(load().mw_allgather_step(self._h, _ptr(shard), C.c_int64(shard_bytes), _ptr(send_buf), _ptr(desc),
                                        _ptr(stats), _ptr(peer_shards), _ptr(out), _stream()), "mw_allgather_step")

    # ---- relay ---------------------------------------------------------------------------
    def mw_set_forwarding(self, next_hop: np.ndarray, n_hops: int):
        t = np.ascontiguousarray(next_hop, dtype=np.int32)
        _check(load().mw_set_forwarding(self._h, C.c_void_p(t.ctypes.data), C.c_int32(n_hops)), "mw_set_forwarding")

    def mw_relay(self, in_record: torch.Tensor, children: torch.Tensor, child_capacity_rows: int,
                 stats: torch.Tensor):
        _check(load().mw_relay(self._h, _ptr(in_record), _ptr(children), C.c_int64(child_capacity_rows),
                               _ptr(stats), _stream()), "mw_relay")

    def mw_relay_index(self, in_record: torch.Tensor, children: torch.Tensor, child_capacity_rows: int,
                       stats: torch.Tensor):
        _check(load().mw_relay_index(self._h, _ptr(in_record), _ptr(children), C.c_int64(child_capacity_rows),
                                     _ptr(stats), _stream()), "mw_relay_index")

    def mw_relay_copy(self, in_record: torch.Tensor, children: torch.Tensor, stats: torch.Tensor):
        _check(load().mw_relay_copy(self._h, _ptr(in_record), _ptr(children), _ptr(stats), _stream()),
               "mw_relay_copy")

    def mw_relay_copy_index_next(self, in_record: torch.Tensor, children: torch.Tensor, stats: torch.Tensor,
                                 next_ctx: "Context", next_in_record: torch.Tensor, next_children: torch.Tensor,
                                 next_child_capacity_rows: int, next_stats: torch.Tensor):
        _check(load().mw_relay_copy_index_next(self._h, _ptr(in_record), _ptr(children), _ptr(stats), next_ctx._h,
                                               _ptr(next_in_record), _ptr(next_children),
                                               C.c_int64(next_child_capacity_rows), _ptr(next_stats), _stream()),
               "mw_relay_copy_index_next")

    def mw_relay_packets(self, in_record: torch.Tensor, children: torch.Tensor, child_capacity_rows: int,
                         stats: torch.Tensor):
        _check(load().mw_relay_packets(self._h, _ptr(in_record), _ptr(children), C.c_int64(child_capacity_rows),
                                       _ptr(stats), _stream()), "mw_relay_packets")

    def mw_relay_packets_index(self, in_record: torch.Tensor, child_capacity_rows: int, stats: torch.Tensor):
        _check(load().mw_relay_packets_index(self._h, _ptr(in_record), C.c_int64(child_capacity_rows), _ptr(stats),
                                             _stream()), "mw_relay_packets_index")

    def mw_relay_packets_copy(self, in_record: torch.Tensor, children: torch.Tensor, stats: torch.Tensor):
        _check(load().mw_relay_packets_copy(self._h, _ptr(in_record), _ptr(children), _ptr(stats), _stream()),
               "mw_relay_packets_copy")

    def mw_relay_packets_copy_index_next(self, in_record: torch.Tensor, children: torch.Tensor, stats: torch.Tensor,
                                         next_ctx: "Context", next_in_record: torch.Tensor,
                                         next_child_capacity_rows: int, next_stats: torch.Tensor):
        _check(load().mw_relay_packets_copy_index_next(self._h, _ptr(in_record), _ptr(children), _ptr(stats),
                                                       next_ctx._h, _ptr(next_in_record),
                                                       C.c_int64(next_child_capacity_rows), _ptr(next_stats),
                                                       _stream()), "mw_relay_packets_copy_index_next")

    def mw_get_relay_stats(self, stats: torch.Tensor) -> np.ndarray:
        host = np.zeros(1, dtype=RELAY_STATS_DTYPE)
        _check(load().mw_get_relay_stats(self._h, _ptr(stats), C.c_void_p(host.ctypes.data), _stream()),
               "mw_get_relay_stats")
        return host[0]

    # ---- simulation / statistics ---------------------------------------------------------
    def mw_sim_deliver(self, desc, stats, n_tokens, packed, row_src_token, row_topk, dst_rank,
                       desc_out, rows_out, src_token_out, topk_out, counts_out):
        _check(load().mw_sim_deliver(self._h, _ptr(desc), _ptr(stats), C.c_int32(n_tokens), _ptr(packed),
                                     _ptr(row_src_token), _ptr(row_topk), C.c_int32(dst_rank),
                                     _ptr(desc_out), _ptr(rows_out), _ptr(src_token_out), _ptr(topk_out),
                                     _ptr(counts_out), _stream()), "mw_sim_deliver")

    def mw_ctx_set_timing_events(self, kernel: int, ev_start: Optional[torch.cuda.Event],
                                 ev_stop: Optional[torch.cuda.Event]):
        """Events must have been recorded once already (torch creates the handle lazily)."""
        a = C.c_void_p(0 if ev_start is None else ev_start.cuda_event)
        b = C.c_void_p(0 if ev_stop is None else ev_stop.cuda_event)
        _check(load().mw_ctx_set_timing_events(self._h, C.c_int32(kernel), a, b), "mw_ctx_set_timing_events")

    def mw_get_send_stats(self, stats: torch.Tensor) -> np.ndarray:
        host = np.zeros(1, dtype=SEND_STATS_DTYPE)
        _check(load().mw_get_send_stats(self._h, _ptr(stats), C.c_void_p(host.ctypes.data), _stream()),
               "mw_get_send_stats")
        return host[0]

    def mw_get_recv_stats(self, stats: torch.Tensor) -> np.ndarray:
        host = np.zeros(1, dtype=RECV_STATS_DTYPE)
        _check(load().mw_get_recv_stats(self._h, _ptr(stats), C.c_void_p(host.ctypes.data), _stream()),
               "mw_get_recv_stats")
        return host[0]


# ---- buffer helpers (allocation only) ----------------------------------------------------
def peers_table(records: Sequence[dict], device) -> torch.Tensor:
    """Device array of mw_recv_peer records from dicts of device tensors
    {desc, n_desc, n_rows, rows, row_src_token, row_topk}."""
    host = np.zeros(max(len(records), 1), dtype=RECV_PEER_DTYPE)
    for i, r in enumerate(records):
        host[i] = (r["desc"].data_ptr(), r["n_desc"], r["n_rows"], r["rows"].data_ptr(),
                   r["row_src_token"].data_ptr(), r["row_topk"].data_ptr())
    return torch.from_numpy(host.view(np.uint8).reshape(-1)).to(device)


def packets_table(regions: Sequence[torch.Tensor], n_rows: Sequence[int], device) -> torch.Tensor:
    """Device array of mw_recv_packets records from device tensors of packets."""
    host = np.zeros(max(len(regions), 1), dtype=RECV_PACKETS_DTYPE)
    for i, (r, n) in enumerate(zip(regions, n_rows)):
        host[i] = (r.data_ptr(), n, 0)
    return torch.from_numpy(host.view(np.uint8).reshape(-1)).to(device)


class RelayChildren:
    """Output buffers of mw_relay for n_hops children of `capacity` rows each."""

    def __init__(self, ctx: Context, n_hops: int, capacity: int):
        d, n = ctx.device, max(capacity, 1)
        self.n_hops, self.capacity = n_hops, capacity
        self.desc = [torch.zeros((n, DESC_BYTES), dtype=torch.uint8, device=d) for _ in range(n_hops)]
        self.rows = [torch.zeros((n, ctx.row_stride), dtype=torch.uint8, device=d) for _ in range(n_hops)]
        self.row_src_token = [torch.full((n,), -1, dtype=torch.int32, device=d) for _ in range(n_hops)]
        self.row_topk = [torch.zeros((n, ctx.top_k), dtype=torch.int32, device=d) for _ in range(n_hops)]
        host = np.zeros(max(n_hops, 1), dtype=RELAY_CHILD_DTYPE)
        for h in range(n_hops):
            host[h] = (self.desc[h].data_ptr(), self.rows[h].data_ptr(), self.row_src_token[h].data_ptr(),
                       self.row_topk[h].data_ptr())
        self.table = torch.from_numpy(host.view(np.uint8).reshape(-1)).to(d)
        self.stats = torch.zeros(RELAY_STATS_BYTES, dtype=torch.uint8, device=d)

    def record(self, h: int, n_desc: int, n_rows: int) -> dict:
        """Child h as a peer record (for peers_table / a further relay)."""
        return dict(desc=self.desc[h], rows=self.rows[h], row_src_token=self.row_src_token[h],
                    row_topk=self.row_topk[h], n_desc=n_desc, n_rows=n_rows)


class SendBuffers:
    """Outputs of mw_plan + mw_pack for up to n_tokens tokens."""

    def __init__(self, ctx: Context, n_tokens: int):
        d, n = ctx.device, max(n_tokens, 1)
        self.mask = torch.zeros((n, 4), dtype=torch.int64, device=d)
        self.perm = torch.full((n,), -1, dtype=torch.int32, device=d)
        self.desc = torch.zeros((n, DESC_BYTES), dtype=torch.uint8, device=d)
        self.stats = torch.zeros(SEND_STATS_BYTES, dtype=torch.uint8, device=d)
        self.packed = torch.zeros((n, ctx.row_stride), dtype=torch.uint8, device=d)
        self.row_src_token = torch.full((n,), -1, dtype=torch.int32, device=d)
        self.row_topk = torch.zeros((n, ctx.top_k), dtype=torch.int32, device=d)


class RecvBuffers:
    """Outputs of mw_unpack for up to `capacity` output rows."""

    def __init__(self, ctx: Context, capacity: int):
        d, n = ctx.device, max(capacity, 1)
        self.capacity = capacity
        self.out_rows = torch.zeros((n, ctx.x_row_bytes), dtype=torch.uint8, device=d)
        self.out_scales = (torch.zeros((n, ctx.s_row_bytes), dtype=torch.uint8, device=d)
                           if ctx.s_row_bytes else None)
        self.out_src_peer = torch.full((n,), -1, dtype=torch.int32, device=d)
        self.out_src_token = torch.full((n,), -1, dtype=torch.int32, device=d)
        self.expert_offsets = torch.zeros(ctx.n_local + 1, dtype=torch.int64, device=d)
        self.stats = torch.zeros(RECV_STATS_BYTES, dtype=torch.uint8, device=d)
