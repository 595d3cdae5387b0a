"""ctypes front end of the CPU oracle (oracle/mw_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of bench.py.  It imports nothing from the HIP package.
Every function takes and returns plain numpy arrays on the host; the record
layouts (48-byte group descriptor, 1056-byte send statistics) are declared
here independently of the HIP library's header.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

DESC = np.dtype([("mask", "<u8", (4,)), ("row_offset", "<u4"), ("row_count", "<u4"),
                 ("n_dest", "<u4"), ("reserved0", "<u4")])
STATS = np.dtype([("n_rows", "<u4"), ("n_groups", "<u4"), ("multicast_bytes", "<u8"),
                  ("unicast_bytes", "<u8"), ("rows_per_dest", "<u4", (256,)),
                  ("error_flags", "<u4"), ("reserved0", "<u4")])
assert DESC.itemsize == 48 and STATS.itemsize == 1056

OK, ERR_ARG, ERR_EXPERT, ERR_CAPACITY, ERR_INPUT = 0, -1, -2, -3, -4


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__("oracle %s failed with code %d" % (where, code))
        self.code = code


class _RecvPeer(C.Structure):
    _fields_ = [("desc", C.c_void_p), ("n_desc", C.c_uint32), ("n_rows", C.c_uint32),
                ("rows", C.c_void_p), ("row_src_token", C.c_void_p), ("row_topk", C.c_void_p)]


class _RecvPackets(C.Structure):
    _fields_ = [("packets", C.c_void_p), ("n_rows", C.c_uint32), ("reserved0", C.c_uint32)]


class _PeerTokens(C.Structure):
    _fields_ = [("topk", C.c_void_p), ("n_tokens", C.c_int32),
                ("x", C.c_void_p), ("scales", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        for name in ("ref_masks", "ref_plan", "ref_accounting_plain", "ref_pack", "ref_deliver",
                     "ref_unpack", "ref_dispatch_plain", "ref_plan_allgather",
                     "ref_pack_allgather", "ref_unpack_allgather",
                     "ref_relay_child", "ref_relay_accounting", "ref_allgather_split_point",
                     "ref_plan_allgather_split", "ref_unpack_allgather_split",
                     "ref_pack_packets", "ref_deliver_packets", "ref_unpack_packets",
                     "ref_quantize_e4m3_block128", "ref_combine_gather", "ref_relay_packets_child",
                     "ref_relay_packets_child_unmodified", "ref_relay_child_unmodified", "ref_unpack_dedup"):
            getattr(_lib, name).restype = C.c_int
        _lib.ref_packet_header_bytes.restype = C.c_int64
    return _lib


def _p(a: Optional[np.ndarray]):
    return C.c_void_p(0 if a is None else a.ctypes.data)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _bytes2d(a: np.ndarray) -> np.ndarray:
    """View a contiguous [n][...] array as uint8 [n][row_bytes]."""
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(a.shape[0], -1) if a.shape[0] else \
        np.zeros((0, int(np.prod(a.shape[1:])) * a.itemsize), np.uint8)


def _check(rc: int, where: str):
    if rc != OK:
        raise OracleError(rc, where)


# ---------------------------------------------------------------------------
def masks(topk, e2r, n_ranks: int) -> np.ndarray:
    topk, e2r = _i32(topk), _i32(e2r)
    T, K = topk.shape
    m = np.zeros((T, 4), dtype=np.uint64)
    _check(lib().ref_masks(_p(topk), C.c_int32(T), C.c_int32(K), _p(e2r), C.c_int32(len(e2r)),
                           C.c_int32(n_ranks), _p(m)), "ref_masks")
    return m


def plan(topk, e2r, n_ranks: int, row_bytes: int):
    """-> (mask [T][4] u64, perm [N] i32, desc [G] DESC, stats STATS scalar)"""
    topk, e2r = _i32(topk), _i32(e2r)
    T, K = topk.shape
    m = np.zeros((T, 4), dtype=np.uint64)
    perm = np.full(max(T, 1), -1, dtype=np.int32)
    desc = np.zeros(max(T, 1), dtype=DESC)
    st = np.zeros(1, dtype=STATS)
    _check(lib().ref_plan(_p(topk), C.c_int32(T), C.c_int32(K), _p(e2r), C.c_int32(len(e2r)),
                          C.c_int32(n_ranks), C.c_int64(row_bytes), _p(m), _p(perm), _p(desc), _p(st)),
           "ref_plan")
    N, G = int(st["n_rows"][0]), int(st["n_groups"][0])
    return m, perm[:N].copy(), desc[:G].copy(), st[0]


def accounting_plain(topk, e2r, n_ranks: int, row_bytes: int):
    topk, e2r = _i32(topk), _i32(e2r)
    T, K = topk.shape
    mc, uc = C.c_uint64(0), C.c_uint64(0)
    rpd = np.zeros(256, dtype=np.uint32)
    _check(lib().ref_accounting_plain(_p(topk), C.c_int32(T), C.c_int32(K), _p(e2r),
                                      C.c_int32(len(e2r)), C.c_int32(n_ranks), C.c_int64(row_bytes),
                                      C.byref(mc), C.byref(uc), _p(rpd)), "ref_accounting_plain")
    return int(mc.value), int(uc.value), rpd


def pack(x: np.ndarray, scales: Optional[np.ndarray], topk, perm):
    """x: [T][...] payload, scales: [T][...] or None -> (packed u8 [N][rb], src_token [N], row_topk [N][K])"""
    topk, perm = _i32(topk), _i32(perm)
    xb = _bytes2d(x)
    sb = _bytes2d(scales) if scales is not None else None
    xrb = xb.shape[1]
    srb = sb.shape[1] if sb is not None else 0
    N, K = len(perm), topk.shape[1]
    packed = np.zeros((N, xrb + srb), dtype=np.uint8)
    st = np.zeros(N, dtype=np.int32)
    rt = np.zeros((N, K), dtype=np.int32)
    _check(lib().ref_pack(_p(xb), C.c_int64(xrb), _p(sb), C.c_int64(srb), _p(topk), C.c_int32(K),
                          _p(perm), C.c_int32(N), _p(packed), _p(st), _p(rt)), "ref_pack")
    return packed, st, rt


def deliver(desc: np.ndarray, rows: np.ndarray, src_token, row_topk, dst_rank: int):
    """Simulated network: what `dst_rank` receives from this sender."""
    desc = np.ascontiguousarray(desc, dtype=DESC)
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    src_token, row_topk = _i32(src_token), _i32(row_topk)
    G, N = len(desc), rows.shape[0]
    rb, K = rows.shape[1], row_topk.shape[1]
    d2 = np.zeros(max(G, 1), dtype=DESC)
    r2 = np.zeros((max(N, 1), rb), dtype=np.uint8)
    s2 = np.zeros(max(N, 1), dtype=np.int32)
    t2 = np.zeros((max(N, 1), K), dtype=np.int32)
    g_out, n_out = C.c_int32(0), C.c_int32(0)
    _check(lib().ref_deliver(_p(desc), C.c_int32(G), _p(rows), C.c_int64(rb), _p(src_token),
                             _p(row_topk), C.c_int32(K), C.c_int32(dst_rank), _p(d2), _p(r2),
                             _p(s2), _p(t2), C.byref(g_out), C.byref(n_out)), "ref_deliver")
    g, n = g_out.value, n_out.value
    return d2[:g].copy(), r2[:n].copy(), s2[:n].copy(), t2[:n].copy()


def relay_child(desc: np.ndarray, rows: np.ndarray, src_token, row_topk, next_hop, n_hops: int, hop: int,
                update_metadata: bool = True):
    """The child MultiWrite a relay starts towards next hop `hop` (same tuple layout as deliver);
    update_metadata=False: the bitmaps are forwarded as they came (ref_relay_child_unmodified)."""
    desc = np.ascontiguousarray(desc, dtype=DESC)
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    src_token, row_topk, next_hop = _i32(src_token), _i32(row_topk), _i32(next_hop)
    G, N = len(desc), rows.shape[0]
    rb, K = rows.shape[1], row_topk.shape[1]
    d2 = np.zeros(max(G, 1), dtype=DESC)
    r2 = np.zeros((max(N, 1), rb), dtype=np.uint8)
    s2 = np.zeros(max(N, 1), dtype=np.int32)
    t2 = np.zeros((max(N, 1), K), dtype=np.int32)
    g_out, n_out = C.c_int32(0), C.c_int32(0)
    fn = lib().ref_relay_child if update_metadata else lib().ref_relay_child_unmodified
    _check(fn(_p(desc), C.c_int32(G), _p(rows), C.c_int64(rb), _p(src_token),
              _p(row_topk), C.c_int32(K), _p(next_hop), C.c_int32(len(next_hop)),
              C.c_int32(n_hops), C.c_int32(hop), _p(d2), _p(r2), _p(s2), _p(t2),
              C.byref(g_out), C.byref(n_out)), "ref_relay_child")
    g, n = g_out.value, n_out.value
    return d2[:g].copy(), r2[:n].copy(), s2[:n].copy(), t2[:n].copy()


def relay_accounting(desc: np.ndarray, row_bytes: int, next_hop, n_hops: int):
    """(forward_bytes, unicast_bytes, rows_per_hop[n_hops]) of a relay holding `desc`."""
    desc = np.ascontiguousarray(desc, dtype=DESC)
    next_hop = _i32(next_hop)
    fwd, uni = C.c_uint64(0), C.c_uint64(0)
    rph = np.zeros(n_hops, dtype=np.uint32)
    _check(lib().ref_relay_accounting(_p(desc), C.c_int32(len(desc)), C.c_int64(row_bytes), _p(next_hop),
                                      C.c_int32(len(next_hop)), C.c_int32(n_hops), C.byref(fwd),
                                      C.byref(uni), _p(rph)), "ref_relay_accounting")
    return fwd.value, uni.value, rph


PeerBuf = Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]   # (desc, rows, src_token, row_topk)


def unpack(peers: Sequence[PeerBuf], top_k: int, e2r, my_rank: int, x_row_bytes: int,
           s_row_bytes: int, out_capacity_rows: int):
    """-> (out_rows u8 [Q][xrb], out_scales u8 [Q][srb] | None, src_peer [Q], src_token [Q],
           expert_offsets i64 [L+1], n_recv_rows)"""
    e2r = _i32(e2r)
    L = int((e2r == my_rank).sum())
    keep: List[np.ndarray] = []
    arr = (_RecvPeer * max(len(peers), 1))()
    for i, (d, r, s, t) in enumerate(peers):
        d = np.ascontiguousarray(d, dtype=DESC)
        r = np.ascontiguousarray(r, dtype=np.uint8)
        s, t = _i32(s), _i32(t)
        assert r.ndim == 2 and (r.shape[0] == 0 or r.shape[1] == x_row_bytes + s_row_bytes)
        keep += [d, r, s, t]
        arr[i] = _RecvPeer(d.ctypes.data, len(d), r.shape[0], r.ctypes.data, s.ctypes.data, t.ctypes.data)
    cap = max(int(out_capacity_rows), 1)
    out = np.zeros((cap, x_row_bytes), dtype=np.uint8)
    osc = np.zeros((cap, s_row_bytes), dtype=np.uint8) if s_row_bytes else None
    sp = np.full(cap, -1, dtype=np.int32)
    stok = np.full(cap, -1, dtype=np.int32)
    offs = np.zeros(L + 1, dtype=np.int64)
    m = C.c_int64(0)
    _check(lib().ref_unpack(arr, C.c_int32(len(peers)), C.c_int32(top_k), _p(e2r), C.c_int32(len(e2r)),
                            C.c_int32(my_rank), C.c_int64(x_row_bytes), C.c_int64(s_row_bytes),
                            C.c_int64(out_capacity_rows), _p(out), _p(osc), _p(sp), _p(stok), _p(offs),
                            C.byref(m)), "ref_unpack")
    Q = int(offs[L])
    return out[:Q], (osc[:Q] if osc is not None else None), sp[:Q], stok[:Q], offs, int(m.value)


def unpack_dedup(peers: Sequence[PeerBuf], top_k: int, e2r, my_rank: int, x_row_bytes: int,
                 s_row_bytes: int, out_capacity_rows: int):
    """unpack with the end node's de-duplication: inside a peer's region the first row of every
    source token is taken.  -> unpack's tuple with (rows taken, repeats dropped) as its last entry."""
    e2r = _i32(e2r)
    L = int((e2r == my_rank).sum())
    keep: List[np.ndarray] = []
    arr = (_RecvPeer * max(len(peers), 1))()
    for i, (d, r, s, t) in enumerate(peers):
        d = np.ascontiguousarray(d, dtype=DESC)
        r = np.ascontiguousarray(r, dtype=np.uint8)
        s, t = _i32(s), _i32(t)
        keep += [d, r, s, t]
        arr[i] = _RecvPeer(d.ctypes.data, len(d), r.shape[0], r.ctypes.data, s.ctypes.data, t.ctypes.data)
    cap = max(int(out_capacity_rows), 1)
    out = np.zeros((cap, x_row_bytes), dtype=np.uint8)
    osc = np.zeros((cap, s_row_bytes), dtype=np.uint8) if s_row_bytes else None
    sp = np.full(cap, -1, dtype=np.int32)
    stok = np.full(cap, -1, dtype=np.int32)
    offs = np.zeros(L + 1, dtype=np.int64)
    m, dr = C.c_int64(0), C.c_int64(0)
    _check(lib().ref_unpack_dedup(arr, C.c_int32(len(peers)), C.c_int32(top_k), _p(e2r), C.c_int32(len(e2r)),
                                  C.c_int32(my_rank), C.c_int64(x_row_bytes), C.c_int64(s_row_bytes),
                                  C.c_int64(out_capacity_rows), _p(out), _p(osc), _p(sp), _p(stok), _p(offs),
                                  C.byref(m), C.byref(dr)), "ref_unpack_dedup")
    Q = int(offs[L])
    return out[:Q], (osc[:Q] if osc is not None else None), sp[:Q], stok[:Q], offs, (int(m.value), int(dr.value))


PeerTok = Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]     # (topk, x, scales)


def dispatch_plain(peers: Sequence[PeerTok], e2r, my_rank: int, out_capacity_rows: int):
    """Tier 1: the plain definition.  peers[p] = (topk [T][K], x [T][...], scales [T][...] | None)."""
    e2r = _i32(e2r)
    L = int((e2r == my_rank).sum())
    keep = []
    arr = (_PeerTokens * max(len(peers), 1))()
    xrb = srb = 0
    K = 1
    for i, (tk, x, sc) in enumerate(peers):
        tk = _i32(tk)
        xb = _bytes2d(x)
        sb = _bytes2d(sc) if sc is not None else None
        keep += [tk, xb, sb]
        xrb, K = xb.shape[1], tk.shape[1]
        srb = sb.shape[1] if sb is not None else 0
        arr[i] = _PeerTokens(tk.ctypes.data, tk.shape[0], xb.ctypes.data,
                             0 if sb is None else sb.ctypes.data)
    cap = max(int(out_capacity_rows), 1)
    out = np.zeros((cap, xrb), dtype=np.uint8)
    osc = np.zeros((cap, srb), dtype=np.uint8) if srb else None
    sp = np.full(cap, -1, dtype=np.int32)
    stok = np.full(cap, -1, dtype=np.int32)
    offs = np.zeros(L + 1, dtype=np.int64)
    _check(lib().ref_dispatch_plain(arr, C.c_int32(len(peers)), C.c_int32(K), _p(e2r),
                                    C.c_int32(len(e2r)), C.c_int32(my_rank), C.c_int64(xrb),
                                    C.c_int64(srb), C.c_int64(out_capacity_rows), _p(out), _p(osc),
                                    _p(sp), _p(stok), _p(offs)), "ref_dispatch_plain")
    Q = int(offs[L])
    return out[:Q], (osc[:Q] if osc is not None else None), sp[:Q], stok[:Q], offs


# ---------------------------------------------------------------------------
def plan_allgather(n_ranks: int, shard_bytes: int):
    d = np.zeros(1, dtype=DESC)
    st = np.zeros(1, dtype=STATS)
    _check(lib().ref_plan_allgather(C.c_int32(n_ranks), C.c_int64(shard_bytes), _p(d), _p(st)),
           "ref_plan_allgather")
    return d, st[0]


def pack_allgather(shard: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(shard).view(np.uint8).reshape(-1)
    out = np.zeros_like(b)
    _check(lib().ref_pack_allgather(_p(b), C.c_int64(b.size), _p(out)), "ref_pack_allgather")
    return out


def unpack_allgather(shards: Sequence[np.ndarray]) -> np.ndarray:
    bs = [np.ascontiguousarray(s).view(np.uint8).reshape(-1) for s in shards]
    n = bs[0].size
    assert all(b.size == n for b in bs)
    ptrs = (C.c_void_p * len(bs))(*[b.ctypes.data for b in bs])
    out = np.zeros(n * len(bs), dtype=np.uint8)
    _check(lib().ref_unpack_allgather(ptrs, C.c_int32(len(bs)), C.c_int64(n), _p(out)),
           "ref_unpack_allgather")
    return out


def allgather_split_point(shard_bytes: int, w_direct: float, w_relay: float, copies: int) -> int:
    """Bytes of the direct segment for which both paths finish together (multiple of 16)."""
    a = C.c_int64(0)
    _check(lib().ref_allgather_split_point(C.c_int64(shard_bytes), C.c_double(w_direct), C.c_double(w_relay),
                                           C.c_int32(copies), C.byref(a)), "ref_allgather_split_point")
    return a.value


def plan_allgather_split(n_ranks: int, shard_bytes: int, direct_bytes: int):
    d = np.zeros(2, dtype=DESC)
    st = np.zeros(1, dtype=STATS)
    _check(lib().ref_plan_allgather_split(C.c_int32(n_ranks), C.c_int64(shard_bytes), C.c_int64(direct_bytes),
                                          _p(d), _p(st)), "ref_plan_allgather_split")
    return d, st[0]


def unpack_allgather_split(direct: Sequence[np.ndarray], relayed: Sequence[np.ndarray], shard_bytes: int,
                           direct_bytes: int) -> np.ndarray:
    db = [np.ascontiguousarray(s).view(np.uint8).reshape(-1) for s in direct]
    rb = [np.ascontiguousarray(s).view(np.uint8).reshape(-1) for s in relayed]
    assert all(b.size >= direct_bytes for b in db) and all(b.size >= shard_bytes - direct_bytes for b in rb)
    dp = (C.c_void_p * len(db))(*[b.ctypes.data for b in db])
    rp = (C.c_void_p * len(rb))(*[b.ctypes.data for b in rb])
    out = np.zeros(shard_bytes * len(db), dtype=np.uint8)
    _check(lib().ref_unpack_allgather_split(dp, rp, C.c_int32(len(db)), C.c_int64(shard_bytes),
                                            C.c_int64(direct_bytes), _p(out)), "ref_unpack_allgather_split")
    return out


# ---------------------------------------------------------------------------
# packets: bitmap and row metadata embedded in front of every row (Section 6.4)
def packet_header_bytes(top_k: int) -> int:
    return int(lib().ref_packet_header_bytes(C.c_int32(top_k)))


def pack_packets(x: np.ndarray, scales: Optional[np.ndarray], topk, mask: np.ndarray, perm) -> np.ndarray:
    """-> uint8 [N][header_bytes + row_bytes]"""
    topk, perm = _i32(topk), _i32(perm)
    xb = _bytes2d(x)
    sb = _bytes2d(scales) if scales is not None else None
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    K = topk.shape[1]
    pb = packet_header_bytes(K) + xb.shape[1] + (sb.shape[1] if sb is not None else 0)
    out = np.zeros((len(perm), pb), dtype=np.uint8)
    _check(lib().ref_pack_packets(_p(xb), C.c_int64(xb.shape[1]), _p(sb),
                                  C.c_int64(0 if sb is None else sb.shape[1]), _p(topk), C.c_int32(K), _p(mask),
                                  _p(perm), C.c_int32(len(perm)), _p(out)), "ref_pack_packets")
    return out


def deliver_packets(packets: np.ndarray, dst_rank: int) -> np.ndarray:
    packets = np.ascontiguousarray(packets, dtype=np.uint8)
    out = np.zeros_like(packets)
    n = C.c_int64(0)
    _check(lib().ref_deliver_packets(_p(packets), C.c_int64(packets.shape[0]), C.c_int64(packets.shape[1]),
                                     C.c_int32(dst_rank), _p(out), C.byref(n)), "ref_deliver_packets")
    return out[: n.value]


def unpack_packets(peers: Sequence[np.ndarray], top_k: int, e2r, my_rank: int, x_row_bytes: int,
                   s_row_bytes: int, out_capacity_rows: int):
    """peers[p] = uint8 [n_p][packet_bytes].  Same return value as unpack()."""
    e2r = _i32(e2r)
    L = int((e2r == my_rank).sum())
    keep = []
    arr = (_RecvPackets * max(len(peers), 1))()
    for i, pk in enumerate(peers):
        pk = np.ascontiguousarray(pk, dtype=np.uint8)
        keep.append(pk)
        arr[i] = _RecvPackets(pk.ctypes.data, pk.shape[0], 0)
    cap = max(int(out_capacity_rows), 1)
    out = np.zeros((cap, x_row_bytes), dtype=np.uint8)
    osc = np.zeros((cap, s_row_bytes), dtype=np.uint8) if s_row_bytes else None
    sp = np.full(cap, -1, dtype=np.int32)
    stok = np.full(cap, -1, dtype=np.int32)
    offs = np.zeros(L + 1, dtype=np.int64)
    m = C.c_int64(0)
    _check(lib().ref_unpack_packets(arr, C.c_int32(len(peers)), C.c_int32(top_k), _p(e2r), C.c_int32(len(e2r)),
                                    C.c_int32(my_rank), C.c_int64(x_row_bytes), C.c_int64(s_row_bytes),
                                    C.c_int64(out_capacity_rows), _p(out), _p(osc), _p(sp), _p(stok), _p(offs),
                                    C.byref(m)), "ref_unpack_packets")
    Q = int(offs[L])
    return out[:Q], (osc[:Q] if osc is not None else None), sp[:Q], stok[:Q], offs, int(m.value)


# ---------------------------------------------------------------------------
# quantise-in-pack: bf16 rows -> e4m3 codes + one fp32 scale per 128 elements
def quantize_rows(x_bf16: np.ndarray):
    """x_bf16: uint16 [n][H] bit patterns -> (codes uint8 [n][H], scales float32 [n][H/128])."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    n, H = x.shape
    codes = np.zeros((n, H), dtype=np.uint8)
    scales = np.zeros((n, H // 128), dtype=np.float32)
    _check(lib().ref_quantize_e4m3_block128(_p(x), C.c_int64(n), C.c_int32(H), _p(codes), _p(scales)),
           "ref_quantize_e4m3_block128")
    return codes, scales


# ---------------------------------------------------------------------------
# the way back: one row per received row, the sum of its local experts' outputs
def combine_gather(peers: Sequence[PeerBuf], top_k: int, e2r, my_rank: int, y_bf16: np.ndarray,
                   out_src_peer, out_src_token, expert_offsets) -> List[np.ndarray]:
    """peers as for unpack(); y_bf16 uint16 [Q][H] laid out like unpack()'s out_rows.
    -> per peer uint16 [n_rows_p][H]; rows not addressed to my_rank stay zero."""
    e2r = _i32(e2r)
    y = np.ascontiguousarray(y_bf16, dtype=np.uint16)
    H = y.shape[1]
    sp, stok = _i32(out_src_peer), _i32(out_src_token)
    offs = np.ascontiguousarray(expert_offsets, dtype=np.int64)
    keep: List[np.ndarray] = []
    arr = (_RecvPeer * max(len(peers), 1))()
    outs = []
    for i, (d, r, s, t) in enumerate(peers):
        d = np.ascontiguousarray(d, dtype=DESC)
        s, t = _i32(s), _i32(t)
        keep += [d, s, t]
        arr[i] = _RecvPeer(d.ctypes.data, len(d), len(s), 0, s.ctypes.data, t.ctypes.data)
        outs.append(np.zeros((len(s), H), dtype=np.uint16))
    ptrs = (C.c_void_p * max(len(peers), 1))(*[o.ctypes.data for o in outs])
    _check(lib().ref_combine_gather(arr, C.c_int32(len(peers)), C.c_int32(top_k), _p(e2r), C.c_int32(len(e2r)),
                                    C.c_int32(my_rank), C.c_int32(H), _p(y), _p(sp), _p(stok), _p(offs), ptrs),
           "ref_combine_gather")
    return outs


def relay_packets_child(packets: np.ndarray, next_hop, n_hops: int, hop: int, update_metadata: bool = True):
    """-> (child packets of next hop `hop`, packets written by the whole relay step, destinations named);
    update_metadata=False: the kept packets as they arrived (-> child packets only)"""
    packets = np.ascontiguousarray(packets, dtype=np.uint8)
    next_hop = _i32(next_hop)
    out = np.zeros_like(packets)
    n, copies, dests = C.c_int64(0), C.c_uint64(0), C.c_uint64(0)
    if not update_metadata:
        _check(lib().ref_relay_packets_child_unmodified(_p(packets), C.c_int64(packets.shape[0]),
                                                        C.c_int64(packets.shape[1]), _p(next_hop),
                                                        C.c_int32(len(next_hop)), C.c_int32(n_hops), C.c_int32(hop),
                                                        _p(out), C.byref(n)),
               "ref_relay_packets_child_unmodified")
        return out[: n.value].copy()
    _check(lib().ref_relay_packets_child(_p(packets), C.c_int64(packets.shape[0]), C.c_int64(packets.shape[1]),
                                         _p(next_hop), C.c_int32(len(next_hop)), C.c_int32(n_hops), C.c_int32(hop),
                                         _p(out), C.byref(n), C.byref(copies), C.byref(dests)),
           "ref_relay_packets_child")
    return out[: n.value].copy(), copies.value, dests.value
